"""CPU-side checks of the boundary: the library loads without a GPU, exports every symbol that
include/moe.h declares, and its host-only helpers behave (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

from paper_2503_09716_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_static_scratch_size_matches_the_header():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    m = re.search(r"#define\s+MOE_STATIC_WORKSPACE_BYTES\s+\(\(size_t\)(\d+)\s*<<\s*(\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == binding.STATIC_WORKSPACE_BYTES


def test_workspace_bytes_host_logic():
    s = binding.make_shape(4096, 4096, 14336, 8, 2)
    n = binding.workspace_bytes(s)
    R = 4096 * 2
    assert n >= R * 14336 * 2 + R * 4096 * 2          # h + y_perm at least
    assert n % 256 == 0
    # shared experts add their rows of h and the y_shared buffer
    s2 = binding.make_shape(4096, 4096, 14336, 8, 2, num_shared=1)
    assert binding.workspace_bytes(s2) >= n + 4096 * 14336 * 2 + 4096 * 4096 * 2
    # invalid / unsupported shapes report 0
    assert binding.workspace_bytes(binding.make_shape(0, 64, 64, 4, 1)) > 0      # an empty batch is a valid shape
    for bad in [binding.make_shape(-1, 64, 64, 4, 1), binding.make_shape(8, 64, 64, 4, 5),
                binding.make_shape(8, 60, 64, 4, 1), binding.make_shape(8, 64, 72, 4, 1),
                binding.make_shape(8, 64, 64, 300, 1), binding.make_shape(8, 64, 64, 4, 1, num_shared=9)]:
        assert binding.workspace_bytes(bad) == 0


def test_layer_views_rejects_bad_arguments():
    lib = binding.load_library()
    s = binding.make_shape(8, 64, 64, 4, 5)
    p = C.c_void_p()
    assert lib.moe_layer_views(C.byref(s), C.c_void_p(256), C.byref(p), None, None, None) != 0
    s = binding.make_shape(8, 64, 64, 4, 2)
    assert lib.moe_layer_views(C.byref(s), None, C.byref(p), None, None, None) != 0
    assert lib.moe_layer_views(C.byref(s), C.c_void_p(4096), C.byref(p), None, None, None) == 0
    assert p.value == 4096      # topk_idx is the first region of the workspace


def test_null_context_calls_fail_cleanly():
    lib = binding.load_library()
    assert lib.moe_set_option(None, b"xcd_remap", 1) != 0
    assert lib.moe_profile_enable(None, 1) != 0
    assert lib.moe_last_error(None) == b"context is NULL"
    lib.moe_destroy(None)
