"""The C-ABI library loads and exports every symbol include/prism.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2510_15620_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "prism.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(prism_[a-z_0-9]+)\s*\(", src)))


@pytest.fixture(scope="module")
def built():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2510_15620_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(binding.LIB_PATH)


def test_every_declared_symbol_is_exported(built):
    names = _declared()
    assert "prism_select" in names and "prism_create" in names and len(names) >= 15
    for n in names:
        assert hasattr(built, n), n
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_the_header():
    # sizes implied by the header's field lists (natural alignment, LP64)
    assert ctypes.sizeof(binding.prism_model) == 11 * 4
    assert ctypes.sizeof(binding.prism_layer_weights) == 11 * 8
    assert ctypes.sizeof(binding.prism_weights) == 7 * 8
    assert ctypes.sizeof(binding.prism_options) == 8 + 4 * 6 + 8 + 8 + 4 * 6     # six trailing int32
    assert ctypes.sizeof(binding.prism_report) == 3 * 4 + 4 + 10 * 8 + 3 * 8 + 3 * 8 + 4 + 6 * 4 + 4 + 6 * 8 + 6 * 8 + 3 * 8 + 2 * 4 + 4 * 8 + 8 + 8   # kind_mask (int32) + padding, ms_transfers


def test_strerror_and_argument_errors_without_a_gpu(built):
    built.prism_strerror.restype = ctypes.c_char_p
    assert built.prism_strerror(0) == b"ok"
    assert b"invalid" in built.prism_strerror(-1)
    # null arguments are rejected before any HIP call
    assert built.prism_create(None, None, None, None) == binding.EINVAL
    assert built.prism_select(None, None, 0, None, None, 0, 0, None, None, None, None) == binding.EINVAL
    built.prism_destroy(None)


def test_generated_gemm_loop_is_in_sync_with_its_generator():
    """gemm_16_kloop.inc is committed next to the script that writes it; the two must not drift apart."""
    import os
    import subprocess
    import sys
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2510_15620_amd", "csrc")
    out = subprocess.run([sys.executable, os.path.join(csrc, "gen_gemm_kloop.py")], capture_output=True, text=True, check=True).stdout
    assert out == open(os.path.join(csrc, "gemm_16_kloop.inc")).read()


def test_vt_column_mapping_is_the_documented_order(built):
    """Within every group of 16 key positions the transposed-V columns hold the keys in the order 0-3, 8-11, 4-7, 12-15
    (a host function: no GPU is touched)."""
    built.prism_vt_column_of_key.restype = ctypes.c_int32
    built.prism_vt_column_of_key.argtypes = [ctypes.c_int32]
    cols = [built.prism_vt_column_of_key(p) for p in range(48)]
    order = [0, 1, 2, 3, 8, 9, 10, 11, 4, 5, 6, 7, 12, 13, 14, 15]
    held = [cols.index(c) for c in range(48)]                # key found at column c
    assert held == [g * 16 + k for g in range(3) for k in order]
    assert sorted(cols) == list(range(48)) and built.prism_vt_column_of_key(-3) == -3
