"""CPU-only checks of the boundary: the shared library loads and exports every entry point
that include/copyspec.h declares, and the binding's struct layouts match the header."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "copyspec.h")
LIB = os.path.join(ROOT, "paper_2502_08923_amd", "libcopyspec.so")


def declared_symbols():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(cs_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2502_08923_amd.build import build_lib
        build_lib()
    return ctypes.CDLL(LIB)


def test_header_declares_the_named_calls():
    syms = declared_symbols()
    for name in ("cs_find_match", "cs_verify", "cs_decode", "cs_step", "cs_kv_set_len"):
        assert name in syms


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} declared in copyspec.h but not exported"


def test_binding_lists_every_declared_symbol():
    from paper_2502_08923_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()
    binding.load_library()


def test_struct_layouts_match_header():
    from paper_2502_08923_amd import binding
    assert ctypes.sizeof(binding.cs_model_cfg) == 12 * 4
    assert ctypes.sizeof(binding.cs_layer_weights) == 12 * 8
    assert ctypes.sizeof(binding.cs_weights) == 4 * 8
    assert ctypes.sizeof(binding.cs_stats) == 4 * 8
    assert ctypes.sizeof(binding.cs_merged_stats) == 8 * 8


def test_version_and_error_strings_without_gpu(lib):
    lib.cs_version.restype = ctypes.c_char_p
    lib.cs_last_error.restype = ctypes.c_char_p
    assert b"copyspec" in lib.cs_version()
    assert isinstance(lib.cs_last_error(), bytes)


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_08923_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2502_08923_amd" not in text and "libcopyspec" not in text
