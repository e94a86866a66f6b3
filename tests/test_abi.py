"""The C-ABI library loads on a machine without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2501_15348_amd import build, reinc

    if not os.path.exists(reinc.LIB_PATH):
        build.build_library()
    return reinc.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "reinc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(reinc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 20
    for name in names:
        assert hasattr(lib, name), f"{name} declared in reinc.h but not exported"


def test_struct_sizes_match_header(lib):
    from paper_2501_15348_amd import reinc

    # a wrong struct_size must be rejected without touching the device
    cfg = reinc.Config()
    cfg.struct_size = 4
    h = ctypes.c_void_p()
    assert lib.reinc_create(ctypes.byref(h), ctypes.byref(cfg)) == reinc.E_ARG
    assert not h.value
    assert lib.reinc_version().startswith(b"reinc-hip")


def test_bad_config_reports_text(lib):
    from paper_2501_15348_amd import reinc

    cfg = reinc.Config()
    cfg.struct_size = ctypes.sizeof(reinc.Config)
    cfg.num_nodes = 0
    h = ctypes.c_void_p()
    rc = lib.reinc_create(ctypes.byref(h), ctypes.byref(cfg))
    assert rc == reinc.E_ARG and h.value
    assert b"num_nodes" in lib.reinc_last_error(h)
    lib.reinc_destroy(h)
