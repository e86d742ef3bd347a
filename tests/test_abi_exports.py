"""Host checks of the boundary: the built library exports every function include/als.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "als.h")
LIB = os.path.join(ROOT, "paper_2112_02194_amd", "libals.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(als_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_named_entry_points():
    names = declared_functions()
    for required in ("als_gramian", "als_solve_rows", "als_epoch", "als_loss", "als_create", "als_destroy"):
        assert required in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"libals.so does not export {name}"


def test_binding_lists_the_same_names():
    from paper_2112_02194_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()


def test_strerror_needs_no_gpu():
    from paper_2112_02194_amd import binding
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    lib = binding.load_library()
    assert lib.als_strerror(0) == b"ok"
    assert b"positive definite" in lib.als_strerror(binding.ALS_ENOTSPD)


def test_binding_fails_loudly_without_gpu():
    import torch
    from paper_2112_02194_amd import binding
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(RuntimeError):
        binding.Context(0)
