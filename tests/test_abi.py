"""The C-ABI library builds, loads, and exports every entry point that
include/rsvd.h declares (no compute calls here: no GPU needed)."""
import os
import re

from paper_2110_03423_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rsvd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rsvd_[a-z0-9_]+)\s*\(", text)))


def _lib():
    if not os.path.exists(binding.library_path()):
        from paper_2110_03423_amd import build
        build.build_library()
    return binding.load_library()


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert "rsvd_run" in names and len(names) >= 14
    lib = _lib()
    for name in names:
        assert hasattr(lib, name), name
        assert name in binding.PROTOTYPES, f"{name} has no Python prototype"
    assert sorted(binding.PROTOTYPES) == names


def test_status_strings_and_host_only_argument_checks():
    lib = _lib()
    assert lib.rsvd_status_string(0) == b"success"
    assert b"Jacobi" in lib.rsvd_status_string(2)
    assert lib.rsvd_status_string(-4) == b"invalid argument"
    # null context is rejected before anything touches a device
    assert lib.rsvd_workspace_bytes(None, 0, 10, 10, 2, 2, 1, 2, None) == -1
    assert lib.rsvd_run(None, None, 0, 2, 10, 10, None, 10, 2, 2, 1, 0, None, None, 0, None, 0, None, 0, None) == -1
