"""GPU test of bnn_net_forward_static (the entry point that allocates nothing): its output against
bnn_net_forward's on the same inputs, two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import host, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bnn():
    import paper_2006_16578_amd as b
    b.load()
    return b


def test_static_forward_matches_forward_two_calls(bnn):
    lib = bnn.load()
    assert lib.bnn_static_workspace_init() == 0
    # binarized MLP (integer scores: bit-exact), larger batch first, then a smaller one on the same buffer
    params = wl.mlp_params()
    net = bnn.Net()
    net.input_u8(784, params["in_thr"])
    for l in range(4):
        net.add_fc(to_dev(params["W"][l]), to_dev(params["thr"][l]) if l < 3 else None, params["K"][l])
    for batch in (1024, 37):
        x = to_dev(wl.mlp_images(batch))
        want = host(net.forward(x))
        out = torch.full((batch, 10), -12345, dtype=torch.int32, device="cuda")
        got = host(net.forward_static(x, out=out))
        assert np.array_equal(got, want), "MLP batch %d" % batch
    # a residual network with an fp32 first and last layer (same kernels in the same order: equal floats), a
    # larger and then a smaller batch
    blocks = ((64, 64, 1), (64, 96, 2), (96, 96, 1), (96, 128, 2))
    p = wl.resnet18_params(blocks=blocks, classes=13, config=95)
    rnet = bnn.Net()
    rnet.input_conv_f32(to_dev(p["stem_w"]), to_dev(p["stem_thr"]), 32, 32, 4, 3)
    for blk in p["blocks"]:
        rnet.add_block(to_dev(blk["W1"]), to_dev(blk["thr1"]), to_dev(blk["W2"]), to_dev(blk["thr2"]),
                       to_dev(blk["Wd"]) if "Wd" in blk else None, blk["cin"], blk["cout"], blk["stride"])
    rnet.add_head_f32(to_dev(p["fc_w"]))
    for batch in (9, 2):
        x = to_dev(wl.resnet18_input(batch, hw=32, config=95))
        want = host(rnet.forward(x))
        got = host(rnet.forward_static(x))
        tol = 1e-4 * np.maximum(np.abs(want), np.sqrt((want.astype(np.float64) ** 2).mean()))
        assert (np.abs(got - want) <= tol).all(), "ResNet batch %d" % batch
        assert np.array_equal(got, want), "ResNet batch %d: same kernels must give the same floats" % batch
    # the MLP again after another network has used the buffer
    x = to_dev(wl.mlp_images(8))
    assert np.array_equal(host(net.forward_static(x)), host(net.forward(x)))


def test_static_forward_rejects_what_does_not_fit(bnn):
    params = wl.mlp_params()
    net = bnn.Net()
    net.input_u8(784, params["in_thr"])
    for l in range(4):
        net.add_fc(to_dev(params["W"][l]), to_dev(params["thr"][l]) if l < 3 else None, params["K"][l])
    batch = 1 << 17
    assert net.workspace_bytes(batch) > (32 << 20)
    x = torch.zeros((batch, 784), dtype=torch.uint8, device="cuda")
    out = torch.empty((batch, 10), dtype=torch.int32, device="cuda")
    with pytest.raises(bnn.BnnError) as e:
        net.forward_static(x, out=out)
    assert e.value.status == -5
    # within the limit it still runs
    assert net.workspace_bytes(65536) <= (32 << 20)
