"""CPU-side checks of the boundary: the HIP library builds into the tree, loads, and exports
every entry point that include/loopserve.h declares (no compute without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2507_13681_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.LIB):
        build.build_library()
    return binding.load_library()


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names.update(re.findall(r"\b(ls_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_exported(lib):
    names = _declared()
    assert {"ls_score", "ls_select", "ls_sparse_prefill", "ls_kv_compress", "ls_create", "ls_destroy",
            "ls_last_error", "ls_workspace_bytes", "ls_poll_status", "ls_debug_set_walk_spin_limit"} <= set(names)
    raw = ctypes.CDLL(build.LIB)
    for n in names:
        assert hasattr(raw, n), n


def test_workspace_bytes_is_host_only(lib):
    s = binding.make_shape(1, 32, 8, 128, 32768, 10923, 64, "bf16")
    b = binding.workspace_bytes(s, 2048)
    # ls_select alone needs keys and two index arrays per (list, head, position) = 24 bytes
    assert 24 * 32 * 32768 <= b < 2 ** 31
    bad = binding.make_shape(1, 32, 7, 128, 32768, 10923, 64, "bf16")       # Hq % Hkv != 0
    assert binding.workspace_bytes(bad) == 0
    bad = binding.make_shape(1, 32, 8, 96, 32768, 10923, 64, "bf16")        # unsupported head dim
    assert binding.workspace_bytes(bad) == 0


def test_struct_layout_matches_header():
    assert ctypes.sizeof(binding.LsShape) == 48
    assert binding.LsShape.n.offset == 16 and binding.LsShape.w.offset == 32 and binding.LsShape.scale.offset == 40


def test_product_path_does_not_import_oracle():
    """The package must not reach into oracle/ (the oracle is test infrastructure)."""
    pkg = os.path.join(ROOT, "paper_2507_13681_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|ls_oracle|lso_", src, flags=re.M), f
