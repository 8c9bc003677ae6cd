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


def test_header_compiles_as_c99_and_the_config_struct_matches_the_binding(tmp_path):
    """include/h1bkv.h is compiled by a C compiler (not read with regular expressions): size and field offsets of
    h1bkv_config as the compiler lays them out must be those of the ctypes mirror in the binding, in the same order."""
    import subprocess
    fields = [name for name, _ in B.h1bkv_config._fields_]
    src = tmp_path / "probe.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "h1bkv.h"', 'int main(void) {',
             '  printf("sizeof %zu\\n", sizeof(h1bkv_config));']
    lines += [f'  printf("{f} %zu %zu\\n", offsetof(h1bkv_config, {f}), sizeof(((h1bkv_config *)0)->{f}));' for f in fields]
    lines += ['  printf("enum %d %d %d %d\\n", H1BKV_K_COUNT, H1BKV_ENODEVICE, H1BKV_F16, H1BKV_DEVICE_NONE);', '  return 0;', '}']
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.dirname(HEADER), str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    assert out[0] == f"sizeof {ctypes.sizeof(B.h1bkv_config)}"
    for line, f in zip(out[1:], fields):
        desc = getattr(B.h1bkv_config, f)
        assert line == f"{f} {desc.offset} {desc.size}", (line, desc.offset, desc.size)
    assert out[1 + len(fields)] == f"enum 5 {B.H1BKV_ENODEVICE} {B.H1BKV_F16} {B.H1BKV_DEVICE_NONE}"
    # every field the header declares is mirrored (a field added to the header only would shift nothing before it)
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    body = re.search(r"typedef struct \{(.*?)\} h1bkv_config;", text, re.S).group(1)
    declared = [n.strip() for decl in body.split(";") if decl.strip() for n in decl.strip().split(None, 1)[1].split(",")]
    assert declared == fields
