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


def test_kernel_choice_is_host_logic():
    # which kernel variant a shape gets is decided on the host: no device needed to ask
    import paper_2006_16578_amd as b
    assert b.bmm_kernel_name(16384, 16384, 16384) == "mfma_fp4_bmm_xlds_wg256x256"
    assert b.bmm_kernel_name(4096, 4096, 4096) == "mfma_fp4_bmm_xlds_wg256x256"        # 256 tiles: one per compute unit
    assert b.bmm_kernel_name(2048, 2048, 2048) == "mfma_fp4_bmm_lds_wg128x128"         # too few 256 x 256 tiles
    assert b.bmm_kernel_name(8, 4096, 4096) == "mfma_fp4_bmm_skinny_m32"               # at most 128 rows: K split over waves
    assert b.bmm_kernel_name(128, 4096, 4096) == "mfma_fp4_bmm_skinny_m128"
    assert b.bmm_kernel_name(129, 4096, 4096) == "mfma_fp4_bmm_wg64x64"
    assert b.bmm_kernel_name(4096, 4096, 4096, b.PATH_VALU) == "valu_xor_popc_bmm"
    # a short-K matrix product with int32 output moves more bytes than it multiplies: small tiles
    assert b.bmm_kernel_name(8192, 8192, 256, int32_out=True) == "mfma_fp4_bmm_wg64x64"
    assert b.bmm_kernel_name(8192, 8192, 256) != "mfma_fp4_bmm_wg64x64"
    # the graded convolution shape: 3x3, stride 1, few channels -> filters resident in LDS, wave-private patches
    assert b.bconv_kernel_name(128, 56, 56, 128, 128, 3, 1, 1) == "mfma_fp4_conv3x3_patch_wave64x128"
    assert b.bconv_kernel_name(128, 56, 56, 128, 128, 3, 1, 1, int32_out=True) == "mfma_fp4_conv3x3_patch_wave64x128"
    assert b.bconv_kernel_name(128, 56, 56, 64, 64, 3, 1, 1) == "mfma_fp4_conv3x3_patch_wave64x64"
    # stride 2, 64 -> 128 channels, bits out: the same kernel with the lane bases twice as far apart
    assert b.bconv_kernel_name(128, 56, 56, 64, 128, 3, 2, 1) == "mfma_fp4_conv3x3s2_patch_wave64x128"
    # the same layers at a small batch, with int32 sums at stride 2, or with more channels: the direct kernel's tiles
    assert b.bconv_kernel_name(2, 56, 56, 128, 128, 3, 1, 1) == "mfma_fp4_conv_wg64x64"
    assert b.bconv_kernel_name(128, 56, 56, 64, 128, 3, 2, 1, int32_out=True) == "mfma_fp4_conv_wg256x128"
    assert not b.bconv_kernel_name(16, 56, 56, 64, 128, 3, 2, 1).startswith("mfma_fp4_conv3x3")     # too few tiles for it
    assert b.bconv_kernel_name(128, 28, 28, 256, 256, 3, 1, 1) == "mfma_fp4_conv_wg256x128"
    # long K goes through LDS
    assert b.bconv_kernel_name(16, 64, 64, 2048, 2048, 3, 1, 1) == "mfma_fp4_conv_lds_wg256x128"
    assert b.bmm_kernel_name(0, 1, 1) == "invalid" and b.bconv_kernel_name(1, 2, 2, 32, 1, 5, 1, 0) == "invalid"


def test_net_workspace_plan():
    # the workspace of a chain grows with the batch and covers residual slots, the first layer's expanded weights
    # and the pooled sums of a head
    import paper_2006_16578_amd as b
    lib = b.load()

    def ws(build, batch):
        net = ctypes.c_void_p()
        assert lib.bnn_net_create(ctypes.byref(net)) == 0
        build(net)
        n = ctypes.c_size_t()
        assert lib.bnn_net_workspace_bytes(net, batch, ctypes.byref(n)) == 0
        assert lib.bnn_net_destroy(net) == 0
        return n.value

    dummy = ctypes.c_void_p(256)            # pointers are only stored by the add calls

    def mlp(net):
        assert lib.bnn_net_input_u8(net, 784, 127) == 0
        assert lib.bnn_net_add_fc(net, dummy, dummy, 784, 1024) == 0
        assert lib.bnn_net_add_fc(net, dummy, None, 1024, 10) == 0

    def resnet(net):
        assert lib.bnn_net_input_conv_f32(net, dummy, dummy, 32, 32, 3, 64, 7, 4, 3) == 0
        assert lib.bnn_net_add_block(net, dummy, dummy, dummy, dummy, None, 64, 64, 1, 0) == 0
        assert lib.bnn_net_add_block(net, dummy, dummy, dummy, dummy, dummy, 64, 128, 2, 0) == 0
        assert lib.bnn_net_add_head_f32(net, dummy, 10) == 0

    assert ws(mlp, 8) < ws(mlp, 1024)
    small, big = ws(resnet, 2), ws(resnet, 64)
    assert small < big
    # at least: two residual slots of 16-bit sums for the largest block output, and its bits twice
    assert big >= 2 * 64 * 8 * 8 * 64 * 2 + 2 * 64 * 8 * 8 * 8


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
