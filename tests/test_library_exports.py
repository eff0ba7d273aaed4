"""The C-ABI library loads and exports every symbol include/april.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "april.h")
LIB = os.path.join(ROOT, "paper_2509_18521_amd", "libapril.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(april_[a-z_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2509_18521_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def test_header_declares_the_three_north_star_calls():
    fns = declared_functions()
    for name in ("april_init", "april_rollout_step", "april_resume"):
        assert name in fns


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_symbols():
    from paper_2509_18521_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()


def test_struct_sizes_match_header_layout():
    from paper_2509_18521_amd import binding as b
    # 7+3+1 int32, 2 float, int32, (pad) int64, 2 int32, 2 int32, float, (pad) uint64, 2 int32, pointer
    assert ctypes.sizeof(b.april_model_cfg) == 128
    assert ctypes.sizeof(b.april_request) == 48
    assert ctypes.sizeof(b.april_tensor) == 32
    assert ctypes.sizeof(b.april_partial) == 72
