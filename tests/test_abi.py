"""CPU-only checks of the boundary: the library loads and exports every symbol include/bnn.h
declares; argument validation that needs no GPU returns the documented codes."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "bnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bnn_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header():
    import paper_2006_16578_amd as b
    lib = b.load()
    syms = declared_symbols()
    assert len(syms) >= 25
    for s in syms:
        assert hasattr(lib, s), s
    assert sorted(b.EXPORTS) == syms


def test_status_strings_and_null_checks():
    import paper_2006_16578_amd as b
    lib = b.load()
    assert lib.bnn_version() >= 100
    assert lib.bnn_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert lib.bnn_status_string(code) not in (b"ok", b"unknown status")
    # validation happens before any device call
    assert lib.bnn_bmm(None, None, None, 1, 1, 1, 4, 4, 1, None) == -1
    assert lib.bnn_bconv(None, None, None, 1, 1, 1, 1, 1, 1, 1, 0, 0, None) == -1
    net = ctypes.c_void_p()
    assert lib.bnn_net_create(ctypes.byref(net)) == 0
    assert lib.bnn_net_add_fc(net, None, None, 8, 8) == -1
    assert lib.bnn_net_input_u8(net, 784, 127) == 0
    assert lib.bnn_net_input_u8(net, 784, 127) == -1          # only one input layer
    n = ctypes.c_size_t()
    assert lib.bnn_net_workspace_bytes(net, 8, ctypes.byref(n)) == 0 and n.value > 0
    assert lib.bnn_net_destroy(net) == 0
