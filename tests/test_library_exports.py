"""The C-ABI library builds, loads and exports every symbol the public header declares.
No compute calls: this runs without a GPU."""
import ctypes
import os
import re

import pytest

from paper_2504_03702_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2504_03702_amd import build
        build.build_library(verbose=False)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "preserve.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ps_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert declared_functions() == sorted(binding.EXPORTS)


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_host_only_calls(lib):
    assert lib.ps_strerror(0) == b"ok"
    assert lib.ps_strerror(-5).startswith(b"workspace")
    assert lib.ps_anticipate_workspace_bytes(4096, 256, 600) > 0
    assert lib.ps_anticipate_workspace_bytes(-1, 256, 600) == 0
    assert lib.ps_anticipate_workspace_bytes(10, 4, 10_000_000) == 0      # a row does not fit LDS
    assert lib.ps_workspace_bytes(None, 10, 1) == 0
    out = ctypes.c_void_p()
    assert lib.ps_model_load(b"/nonexistent/model.bin", 0, ctypes.byref(out)) == -2
    assert lib.ps_model_load(None, 0, ctypes.byref(out)) == -1


def test_bad_model_files_are_rejected(lib, tmp_path):
    from paper_2504_03702_amd import workloads as wl
    out = ctypes.c_void_p()
    p = tmp_path / "junk.bin"
    p.write_bytes(b"not a model" * 10)
    assert lib.ps_model_load(os.fsencode(str(p)), 0, ctypes.byref(out)) == -3
    cfg = wl.MODELS["tiny"]
    good = tmp_path / "tiny.bin"
    wl.write_model(str(good), cfg, wl.make_weights(cfg, 0))
    raw = good.read_bytes()
    trunc = tmp_path / "trunc.bin"
    trunc.write_bytes(raw[:-4])
    assert lib.ps_model_load(os.fsencode(str(trunc)), 0, ctypes.byref(out)) == -3
