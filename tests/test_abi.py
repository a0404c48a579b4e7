"""The C-ABI library loads on a CPU-only host and exports every entry point the header
declares (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def libpath():
    from paper_2410_13229_amd import build as b
    from paper_2410_13229_amd.binding import lib_path

    if not os.path.exists(lib_path()):
        b.build()
    return lib_path()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "quamba.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(quamba_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("quamba_calibrate", "quamba_mixer_prefill", "quamba_mixer_decode", "quamba_workspace_bytes",
                 "quamba_gemm_i8", "quamba_scan_prefill", "quamba_hadamard_quant", "quamba_conv_silu_quant"):
        assert must in names


def test_library_exports_every_declared_symbol(libpath):
    lib = ctypes.CDLL(libpath)
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, missing


def test_binding_covers_every_declared_symbol(libpath):
    import paper_2410_13229_amd as Q

    Q.lib()
    missing = [n for n in declared_functions() if not hasattr(Q, n)]
    assert not missing, missing


def test_host_only_queries(libpath):
    """Size queries and argument checks run on the host without touching a GPU."""
    import paper_2410_13229_amd as Q
    import workloads as W

    c1 = W.CONFIGS["c1"]
    assert Q.quamba_workspace_bytes(c1, 1, 2048) > 2048 * (2560 + 2 * 5120 + 5 * 5120)
    assert Q.quamba_workspace_bytes(c1, 64, 1) > 0
    assert Q.quamba_scan_workspace_bytes(1, 2048, 5120) > 0
    assert Q.quamba_calibrate_workspace_bytes(c1, 4, 256) > 0
    bad = W.tiny_config(d_inner=112)  # 7 * 16: no Hadamard order
    assert Q.quamba_workspace_bytes(bad, 1, 8) == 0
    assert "d_inner" in Q.quamba_last_error()
    with pytest.raises(Q.QuambaError) as e:
        Q.quamba_hadamard_quant(None, 1, 128, 1.0, None, None)
    assert e.value.code == -1
