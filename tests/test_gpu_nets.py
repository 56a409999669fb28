"""GPU parity: the layer-chained forwards (bnn_net_*) against the oracle's compositions."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import host, to_dev, words
from oracle import nets

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bnn():
    import paper_2006_16578_amd as b
    b.load()
    return b


def build_mlp(bnn, params):
    net = bnn.Net()
    net.input_u8(params["dims"][0], params["in_thr"])
    nl = len(params["W"])
    for l in range(nl):
        thr = to_dev(params["thr"][l]) if l < nl - 1 else None
        net.add_fc(to_dev(params["W"][l]), thr, params["K"][l])
    return net


@pytest.mark.parametrize("batch", [8, 1024, 37])
@pytest.mark.parametrize("path", [0, 1, 2])
def test_mlp(bnn, orc, batch, path):
    params = wl.mlp_params()
    imgs = wl.mlp_images(batch)
    ref, hidden = nets.mlp_forward(imgs, params, keep=True)
    net = build_mlp(bnn, params)
    scores = host(net.forward(to_dev(imgs), path=path))
    for l in range(3):
        assert np.array_equal(words(net.layer_bits(l + 1)), hidden[l]), "hidden layer %d" % l
    assert np.array_equal(scores, ref)


def build_resnet(bnn, p, hw, pad_mode=0):
    net = bnn.Net()
    net.input_conv_f32(to_dev(p["stem_w"]), to_dev(p["stem_thr"]), hw, hw, 4, 3)
    for blk in p["blocks"]:
        net.add_block(to_dev(blk["W1"]), to_dev(blk["thr1"]), to_dev(blk["W2"]), to_dev(blk["thr2"]),
                      to_dev(blk["Wd"]) if "Wd" in blk else None, blk["cin"], blk["cout"], blk["stride"], pad_mode)
    net.add_head_f32(to_dev(p["fc_w"]))
    return net


def first_layer_values(bnn, xd, w, thr, stride, pad):
    """fp32 output of a real-weight first layer from the kernel bnn_net_forward runs for it: the bf16 split
    kernel with six term products, or the fp32 matrix-core kernel when the filter bank does not fit it."""
    try:
        _, y = bnn.conv_f32_split_thr(xd, w, thr, stride, pad, want_f32=True, products=6)
    except bnn.BnnError as e:
        if e.status != -3:
            raise
        _, y = bnn.conv_f32_thr(xd, w, thr, stride, pad, want_f32=True)
    return y


def check_resnet(bnn, orc, p, x, hw, path, tier, pad_mode=0):
    """Protocol for a network whose first layer is fp32: the stem output must match within
    1e-4 * max(|o|, rms(o)); a stem bit may differ from the oracle's only where the oracle's value
    is that close to the threshold; the oracle's binarized chain is then run from the GPU's stem
    bits and every later bit tensor must match exactly; logits within the same fp32 tolerance."""
    xd = to_dev(x)
    net = build_resnet(bnn, p, hw, pad_mode)
    logits = host(net.forward(xd, path=path))
    stem_bits_gpu = words(net.layer_bits(0)).reshape(x.shape[0], hw // 4, hw // 4, -1)
    # fp32 stem values, from the kernel the layer chain runs (bf16 x 3 split, six term products)
    y = first_layer_values(bnn, xd, to_dev(p["stem_w"]), to_dev(p["stem_thr"]), 4, 3)
    stem_ref = orc.conv_f32(x, p["stem_w"], 4, 3)
    tol = 1e-4 * np.maximum(np.abs(stem_ref), np.sqrt((stem_ref.astype(np.float64) ** 2).mean()))
    err = np.abs(host(y) - stem_ref)
    print("stem: max |gpu - oracle| = %.3e, max error / tolerance = %.3e" % (err.max(), (err / tol).max()), flush=True)
    assert (err <= tol).all()
    ref_bits = orc.pack_f32(stem_ref, p["stem_thr"])
    diff = stem_bits_gpu ^ ref_bits
    ndiff = 0
    if diff.any():
        # every differing bit must belong to a value inside the tolerance of its threshold
        C = p["stem_w"].shape[0]
        d = orc.unpack_pm1(diff.reshape(-1, diff.shape[-1]), C).reshape(stem_ref.shape) > 0
        assert (np.abs(stem_ref - p["stem_thr"])[d] <= tol[d]).all()
        ndiff = int(d.sum())
    print("stem bits that differ from the oracle's (all inside the fp32 tolerance): %d of %d" % (ndiff, stem_ref.size),
          flush=True)
    tr = nets.resnet18_forward(x, p, stem_bits=stem_bits_gpu, tier=tier, keep=True, pad_mode=pad_mode)
    for b in range(len(p["blocks"])):
        got = words(net.layer_bits(b + 1)).reshape(tr["y%d" % b].shape)
        assert np.array_equal(got, tr["y%d" % b]), "block %d output bits" % b
    ref_logits = tr["logits"]
    tol = 1e-4 * np.maximum(np.abs(ref_logits), np.sqrt((ref_logits.astype(np.float64) ** 2).mean()))
    assert (np.abs(logits - ref_logits) <= tol).all()


@pytest.mark.parametrize("path", [1, 2])
def test_resnet_small(bnn, orc, path):
    blocks = ((64, 64, 1), (64, 96, 2), (96, 96, 1), (96, 128, 2))
    p = wl.resnet18_params(blocks=blocks, classes=13, config=95)
    x = wl.resnet18_input(3, hw=32, config=95)
    check_resnet(bnn, orc, p, x, 32, path, tier=0)


@pytest.mark.parametrize("pad_mode", [0, 1])
@pytest.mark.parametrize("widths", [(64, 80, 80, 96), (64, 64, 128, 128)])
def test_resnet_small_widths_and_padding(bnn, orc, widths, pad_mode):
    # residual chains with channel counts that are not multiples of 32 (row-major 16-bit sums, pad bits inside the
    # last word of a pixel) and with multiples of 32 (blocked sums), in both padding conventions; 5 images of 40x40
    # make ragged 32-row blocks at every resolution
    a, b, c, d = widths
    blocks = ((64, a, 1), (a, b, 2), (b, c, 1), (c, d, 2), (d, d, 1))
    p = wl.resnet18_params(blocks=blocks, classes=21, config=96)
    x = wl.resnet18_input(5, hw=40, config=96)
    check_resnet(bnn, orc, p, x, 40, 0, tier=0, pad_mode=pad_mode)


@pytest.mark.parametrize("seed", [301, 302, 303, 304, 305, 306])
def test_resnet_random_chains(bnn, orc, seed):
    # random residual chains: widths on and off multiples of 32, stride-1 and stride-2 blocks with and without a
    # 1x1 shortcut, random batch and image size, both padding conventions
    rng = np.random.default_rng(seed)
    widths = [int(rng.choice([32, 64, 80, 96, 128, 160])) for _ in range(5)]
    blocks, cin = [], widths[0]
    for b in range(int(rng.integers(3, 6))):
        cout = cin if rng.random() < 0.5 else int(rng.choice(widths))
        stride = 2 if (cout != cin and rng.random() < 0.6) else 1
        blocks.append((cin, cout, stride))
        cin = cout
    hw = int(rng.choice([24, 40, 56]))
    batch = int(rng.integers(1, 7))
    pad_mode = int(rng.integers(0, 2))
    print("chain", blocks, "hw", hw, "batch", batch, "pad_mode", pad_mode, flush=True)
    p = wl.resnet18_params(blocks=tuple(blocks), classes=int(rng.integers(3, 40)), config=seed)
    x = wl.resnet18_input(batch, hw=hw, config=seed)
    check_resnet(bnn, orc, p, x, hw, 0, tier=1, pad_mode=pad_mode)


@pytest.mark.parametrize("blocks,hw,batch,pad_mode", [
    (((64, 64, 1), (64, 64, 1), (64, 96, 2)), 40, 340, 0), (((64, 64, 1), (64, 64, 1), (64, 96, 2)), 40, 340, 1),
    (((128, 128, 1), (128, 128, 1)), 32, 2600, 1)])
def test_resnet_chains_patch_kernel(bnn, orc, blocks, hw, batch, pad_mode):
    # residual chains whose stride-1 layers are large enough for the 3x3 kernel with LDS-resident filters (64- and
    # 128-column forms): bits-only layers, the first residual taken from bits, blocked 16-bit sums in and out, in both
    # padding conventions; 10x10 and 8x8 feature maps, so most 64-pixel tiles cross image rows and images
    H = hw // 4
    cin, cout, _ = blocks[0]
    assert bnn.bconv_kernel_name(batch, H, H, cin, cout, 3, 1, 1).startswith("mfma_fp4_conv3x3_patch")
    p = wl.resnet18_params(blocks=blocks, classes=10, config=97)
    x = wl.resnet18_input(batch, hw=hw, config=97)
    check_resnet(bnn, orc, p, x, hw, 0, tier=1, pad_mode=pad_mode)


def test_resnet18_batch8(bnn, orc):
    p = wl.resnet18_params()
    x = wl.resnet18_input(8)
    check_resnet(bnn, orc, p, x, 224, 0, tier=1)


def test_resnet18_batch256(bnn, orc):
    # the configuration bench.py times (batch 256, automatic path); full comparison of every
    # block's bits against the packed tier-1 oracle chain (tier 1 == tier 0 is pinned on CPU and
    # re-checked above at batch 8 sizes by the small-network test)
    p = wl.resnet18_params()
    x = wl.resnet18_input(256)
    check_resnet(bnn, orc, p, x, 224, 0, tier=1)


@pytest.mark.parametrize("shape", [(9, 7, 7, 512, 1000), (35, 3, 5, 200, 70), (1, 1, 1, 33, 1), (16, 8, 8, 1024, 130), (40, 15, 17, 36, 33)])
def test_head_pooled(bnn, orc, shape):
    # with a pooled-sum output the head runs as two kernels (pool, then FC), without it as one fused kernel
    N, H, W, C, J = shape
    rng = np.random.default_rng(12 + C)
    bits = wl.random_bits(rng, (N, H, W), C)
    w = rng.normal(0, 0.02, size=(J, C)).astype(np.float32)
    pr = orc.sumpool_pm1(bits, C)
    ref = orc.head_fc_f32(pr, w, float(H * W))
    tol = 1e-4 * np.maximum(np.abs(ref), np.sqrt((ref.astype(np.float64) ** 2).mean()))
    y, pooled = bnn.head_f32(to_dev(bits), to_dev(w), C, want_pooled=True)
    assert np.array_equal(host(pooled), pr)
    assert (np.abs(host(y) - ref) <= tol).all()
    y1 = bnn.head_f32(to_dev(bits), to_dev(w), C)
    assert (np.abs(host(y1) - ref) <= tol).all()


@pytest.mark.parametrize("shape", [(2, 21, 19, 3, 5, 7, 4, 3), (1, 9, 9, 1, 1, 3, 1, 1), (3, 16, 12, 4, 70, 5, 2, 2),
                                   (2, 32, 32, 3, 64, 7, 4, 3), (1, 8, 8, 2, 33, 1, 1, 0)])
def test_conv_f32_shapes(bnn, orc, shape):
    N, H, W, C, O, k, st, pad = shape
    rng = np.random.default_rng(sum(shape))
    x = rng.uniform(-1, 1, size=(N, H, W, C)).astype(np.float32)
    w = rng.normal(0, 0.05, size=(O, k, k, C)).astype(np.float32)
    thr = rng.normal(0, 0.05, size=O).astype(np.float32)
    bits, y = bnn.conv_f32_thr(to_dev(x), to_dev(w), to_dev(thr), st, pad, want_f32=True)
    ref = orc.conv_f32(x, w, st, pad)
    tol = 1e-4 * np.maximum(np.abs(ref), np.sqrt((ref.astype(np.float64) ** 2).mean()))
    assert host(y).shape == ref.shape
    assert (np.abs(host(y) - ref) <= tol).all()
    # the bits are exactly the GPU's own fp32 values thresholded, pad bits zero
    assert np.array_equal(words(bits), orc.pack_f32(host(y), thr))


# ------------------------------------------------------------------ max-pooling and the other Table-5 networks
@pytest.mark.parametrize("shape", [(2, 8, 8, 40, 2, 2), (1, 7, 9, 64, 2, 2), (3, 6, 6, 33, 3, 1), (1, 5, 5, 1, 2, 1),
                                   (5, 27, 27, 256, 2, 2), (2, 13, 13, 512, 3, 2), (1, 2, 2, 1024, 2, 2),
                                   (3, 17, 5, 96, 2, 1)])
def test_maxpool_or(bnn, orc, shape):
    N, H, W, C, win, st = shape
    bits = wl.random_bits(np.random.default_rng(sum(shape)), (N, H, W), C)
    got = words(bnn.maxpool_or(to_dev(bits), C, win, st))
    assert np.array_equal(got, orc.maxpool_pm1(bits, C, win, st))


def test_maxpool_or_errors(bnn):
    bits = to_dev(wl.random_bits(np.random.default_rng(0), (1, 4, 4), 32))
    for win, st in ((0, 1), (5, 1), (2, 0)):
        with pytest.raises(bnn.BnnError):
            bnn.maxpool_or(bits, 32, win, st)


def check_cnn(bnn, orc, spec, x, path, tier):
    layers, hw = spec["layers"], spec["in_hw"]
    net = bnn.Net.from_layers(layers, hw)
    xd = to_dev(x)
    scores = host(net.forward(xd, path=path))
    L0 = layers[0]
    if L0["op"] == "bwn":
        _, y = bnn.bwn_conv_thr(xd, to_dev(L0["W"]), to_dev(L0["thr"]), L0["C"], L0["stride"], L0["pad"], want_f32=True)
        ref0 = orc.bwn_conv_f32(x, L0["W"], L0["C"], L0["stride"], L0["pad"])
        cout = L0["W"].shape[0]
    else:
        y = first_layer_values(bnn, xd, to_dev(L0["w"]), to_dev(L0["thr"]), L0["stride"], L0["pad"])
        ref0 = orc.conv_f32(x, L0["w"], L0["stride"], L0["pad"])
        cout = L0["w"].shape[0]
    tol = 1e-4 * np.maximum(np.abs(ref0), np.sqrt((ref0.astype(np.float64) ** 2).mean()))
    err = np.abs(host(y) - ref0)
    print("first layer: max |gpu - oracle| = %.3e, max error / tolerance = %.3e" % (err.max(), (err / tol).max()), flush=True)
    assert (err <= tol).all()
    ref_bits = orc.pack_f32(ref0, L0["thr"])
    bits0 = words(net.layer_bits(0)).reshape(ref_bits.shape)
    diff = bits0 ^ ref_bits
    if diff.any():
        d = orc.unpack_pm1(diff.reshape(-1, diff.shape[-1]), cout).reshape(ref0.shape) > 0
        assert (np.abs(ref0 - L0["thr"])[d] <= tol[d]).all()
        print("first-layer bits inside the fp32 tolerance that differ:", int(d.sum()), flush=True)
    outs = nets.cnn_forward(x, layers, stem_bits=bits0, tier=tier, keep=True)
    for i in range(1, len(layers) - 1):
        got = words(net.layer_bits(i)).reshape(outs[i].shape)
        assert np.array_equal(got, outs[i]), "layer %d (%s) output bits" % (i, layers[i]["op"])
    assert scores.dtype == np.int32 and np.array_equal(scores, outs[-1])


@pytest.mark.parametrize("name,batch,path,tier,first", [
    ("cifar_vgg", 5, 1, 0, "bwn"), ("cifar_vgg", 5, 2, 0, "f32"), ("cifar_vgg", 64, 0, 1, "bwn"),
    ("cifar_resnet14", 5, 1, 0, "f32"), ("cifar_resnet14", 5, 2, 0, "bwn"), ("cifar_resnet14", 64, 0, 1, "bwn"),
    ("alexnet", 3, 2, 1, "f32"), ("alexnet", 16, 0, 1, "bwn"), ("vgg16", 2, 0, 1, "bwn"), ("vgg16", 1, 0, 1, "f32")])
def test_table5_networks(bnn, orc, name, batch, path, tier, first):
    check_cnn(bnn, orc, wl.cnn_layers(name, first=first), wl.cnn_input(name, batch), path, tier)


@pytest.mark.parametrize("shape", [(2, 21, 19, 3, 5, 7, 4, 3), (1, 9, 9, 1, 1, 3, 1, 1), (3, 16, 12, 4, 70, 5, 2, 2),
                                   (2, 32, 32, 3, 64, 7, 4, 3), (1, 8, 8, 2, 33, 1, 1, 0), (2, 32, 32, 3, 128, 3, 1, 1),
                                   (1, 40, 37, 3, 128, 11, 4, 2), (2, 12, 12, 35, 96, 3, 2, 1), (1, 6, 6, 1, 200, 2, 1, 0),
                                   (9, 31, 33, 3, 64, 3, 1, 1)])
def test_bwn_first_layer_shapes(bnn, orc, shape):
    N, H, W, C, O, k, st, pad = shape
    rng = np.random.default_rng(sum(shape) + 1)
    x = rng.uniform(-1, 1, size=(N, H, W, C)).astype(np.float32)
    wb = wl.random_bits(rng, (O, k, k), C)
    thr = rng.normal(0, 1.0, size=O).astype(np.float32)
    bits, y = bnn.bwn_conv_thr(to_dev(x), to_dev(wb), to_dev(thr), C, st, pad, want_f32=True)
    ref = orc.bwn_conv_f32(x, wb, C, st, pad)
    tol = 1e-4 * np.maximum(np.abs(ref), np.sqrt((ref.astype(np.float64) ** 2).mean()))
    assert host(y).shape == ref.shape
    assert (np.abs(host(y) - ref) <= tol).all()
    # far tighter in fact: every product is exact, only the fp32 additions round
    assert np.abs(host(y) - ref).max() <= 2e-6 * max(1.0, np.abs(ref).max()) * np.sqrt(k * k * C)
    assert np.array_equal(words(bits), orc.pack_f32(host(y), thr))
    # bits only (no fp32 output) gives the same words
    assert np.array_equal(words(bnn.bwn_conv_thr(to_dev(x), to_dev(wb), to_dev(thr), C, st, pad)), words(bits))


# 11x11 stride-4 first layers of 3-channel images with at least 4096 rectangles of 4 x 8 output pixels: the kernel with
# wave-private patches (binarized weights: one weight plane); ragged rectangles, ragged and several 64-column tiles,
# images of a single rectangle, odd padding
@pytest.mark.parametrize("shape", [(300, 92, 76, 3, 36, 2), (230, 100, 90, 3, 100, 2), (4200, 11, 13, 3, 64, 2),
                                   (330, 83, 79, 3, 130, 5)])
def test_bwn_first_layer_11x11_wave_kernel(bnn, orc, shape):
    N, H, W, C, O, pad = shape
    k, st = 11, 4
    P, Q = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    assert N * ((P + 3) // 4) * ((Q + 7) // 8) >= 4096
    rng = np.random.default_rng(sum(shape) + 3)
    x = rng.uniform(-1, 1, size=(N, H, W, C)).astype(np.float32)
    wb = wl.random_bits(rng, (O, k, k), C)
    thr = rng.normal(0, 3.0, size=O).astype(np.float32)
    bits, y = bnn.bwn_conv_thr(to_dev(x), to_dev(wb), to_dev(thr), C, st, pad, want_f32=True)
    ref = orc.bwn_conv_f32(x, wb, C, st, pad)
    err = np.abs(host(y) - ref)
    print("bwn 11x11", shape, "max error", float(err.max()), "of rms", float(np.sqrt((ref.astype(np.float64) ** 2).mean())), flush=True)
    assert host(y).shape == ref.shape
    assert (err <= 1e-4 * np.maximum(np.abs(ref), np.sqrt((ref.astype(np.float64) ** 2).mean()))).all()
    assert err.max() <= 2e-6 * max(1.0, np.abs(ref).max()) * np.sqrt(k * k * C)
    assert np.array_equal(words(bits), orc.pack_f32(host(y), thr))
    assert np.array_equal(words(bnn.bwn_conv_thr(to_dev(x), to_dev(wb), to_dev(thr), C, st, pad)), words(bits))
    # integer inputs: every product and every partial sum is exact, so the result equals the oracle's bit for bit
    xi = rng.integers(-2000, 2001, size=(N, H, W, C)).astype(np.float32)
    _, yi = bnn.bwn_conv_thr(to_dev(xi), to_dev(wb), to_dev(thr), C, st, pad, want_f32=True)
    assert np.array_equal(host(yi), orc.bwn_conv_f32(xi, wb, C, st, pad))


def test_bwn_exact_cases(bnn, orc):
    # (a) integer inputs: the three-way bf16 split is exact and sums below 2^24 never round, so the fp32
    # result equals the oracle's bit for bit; (b) isolated values with all 24 significand bits set (at most
    # one non-zero term per output): checks that the split drops no bit
    rng = np.random.default_rng(5)
    wb = wl.random_bits(rng, (40, 5, 5), 3)
    zero = to_dev(np.zeros(40, np.float32))
    x = rng.integers(-30000, 30001, size=(2, 14, 13, 3)).astype(np.float32)
    _, y = bnn.bwn_conv_thr(to_dev(x), to_dev(wb), zero, 3, 2, 2, want_f32=True)
    assert np.array_equal(host(y), orc.bwn_conv_f32(x, wb, 3, 2, 2))
    x = np.zeros((1, 30, 30, 3), np.float32)
    for (h, w, c, v) in ((2, 3, 0, 16777215.0 / 4096), (12, 20, 1, -11184811.0 / 65536), (25, 6, 2, 13421773.0 * 8),
                         (20, 27, 0, 8388609.0 / 2 ** 30)):
        x[0, h, w, c] = v
    _, y = bnn.bwn_conv_thr(to_dev(x), to_dev(wb), zero, 3, 1, 2, want_f32=True)
    ref = orc.bwn_conv_f32(x, wb, 3, 1, 2)
    assert np.abs(ref).max() > 1e7 and np.array_equal(host(y), ref)


# ------------------------------------------------------------------ whole-network persistent kernel (FC chains)
@pytest.mark.parametrize("batch", [8, 37, 1024, 3000])
def test_mlp_persistent(bnn, orc, batch):
    params = wl.mlp_params()
    imgs = wl.mlp_images(batch)
    net = bnn.Net()
    net.input_u8(784, params["in_thr"])
    for l in range(4):
        net.add_fc(to_dev(params["W"][l]), to_dev(params["thr"][l]) if l < 3 else None, params["K"][l])
    ref, hidden = nets.mlp_forward(imgs, params, keep=True)
    x = to_dev(imgs)
    for rep in range(3):                                   # the barrier counter is re-armed on every call
        got = host(net.forward_persistent(x))
        assert not net.persistent_status(), "a barrier gave up in call %d" % rep
        assert np.array_equal(got, ref), "call %d" % rep
    for l in range(3):
        assert np.array_equal(words(net.layer_bits(l + 1)), hidden[l])
    assert np.array_equal(host(net.forward(x)), ref)       # and the per-layer path still agrees


@pytest.mark.parametrize("blocks,hw,batch,pad_mode", [
    (((64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2)), 32, 3, 0),
    (((64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 256, 2), (256, 512, 2), (512, 512, 1)), 64, 2, 1),
    (((128, 128, 1), (128, 128, 1)), 40, 9, 0)])
def test_resnet_persistent(bnn, orc, blocks, hw, batch, pad_mode):
    # residual chains as one persistent kernel (stem and head stay ordinary launches): every block's bits and the
    # logits must equal the per-layer forward's exactly -- the same integer arithmetic, another launch structure --
    # and the per-layer forward is checked against the oracle; repeated calls re-use the uploaded layer table
    p = wl.resnet18_params(blocks=blocks, classes=11, config=98)
    x = wl.resnet18_input(batch, hw=hw, config=98)
    check_resnet(bnn, orc, p, x, hw, 0, tier=1, pad_mode=pad_mode)
    xd = to_dev(x)
    net = build_resnet(bnn, p, hw, pad_mode)
    ref = host(net.forward(xd))
    ref_bits = [words(net.layer_bits(b)) for b in range(len(blocks) + 1)]
    for rep, cap in enumerate((0, 0, 16, 1000)):
        got = host(net.forward_persistent(xd, grid_cap=cap))
        assert not net.persistent_status(), "a barrier gave up in call %d" % rep
        assert np.array_equal(got, ref), "logits, call %d" % rep
        for b in range(len(blocks) + 1):
            assert np.array_equal(words(net.layer_bits(b)), ref_bits[b]), "layer %d, call %d" % (b, rep)
    # another batch through the same net: the table is rebuilt
    x2 = to_dev(wl.resnet18_input(batch + 1, hw=hw, config=99))
    assert np.array_equal(host(net.forward_persistent(x2)), host(net.forward(x2)))


def test_persistent_refuses_what_it_cannot_run(bnn):
    # 96 input channels have no unrolled 3x3 form in the persistent kernel
    p = wl.resnet18_params(blocks=((64, 96, 2), (96, 96, 1)), classes=5, config=98)
    net = build_resnet(bnn, p, 32)
    x = to_dev(wl.resnet18_input(2, hw=32, config=98))
    with pytest.raises(bnn.BnnError) as ei:
        net.forward_persistent(x)
    assert ei.value.status == -3
    assert host(net.forward(x)).shape == (2, 5)            # the per-layer path takes it


def test_persistent_timeout_is_reported(bnn, orc):
    # the time-out path, forced from the host: with a poll limit of zero the first workgroup that finds a barrier
    # incomplete raises the abort flag, every workgroup leaves the kernel normally, and the status call says so;
    # the next ordinary call re-arms the barrier and is exact again
    params = wl.mlp_params()
    imgs = wl.mlp_images(2048)
    net = build_mlp(bnn, params)
    x = to_dev(imgs)
    net.forward_persistent(x, give_up_at_once=True)
    assert net.persistent_status()
    got = host(net.forward_persistent(x))
    assert not net.persistent_status()
    assert np.array_equal(got, nets.mlp_forward(imgs, params))


def test_fc_after_unaligned_spatial_layer_is_refused(bnn):
    # an FC whose operand rows (H*W pixels of ceil(C/32) words) are not a multiple of 128 bits: refused when the
    # workspace is sized, not part-way through the forward
    rng = np.random.default_rng(8)
    net = bnn.Net()
    net.input_conv_f32(to_dev(rng.normal(size=(64, 3, 3, 3)).astype(np.float32)), to_dev(np.zeros(64, np.float32)), 3, 3, 1, 0)
    net.add_fc(to_dev(wl.random_bits(rng, 10, 64, 4)), None, 64)         # 1x1x64: rows of 2 words
    with pytest.raises(bnn.BnnError) as e:
        net.workspace_bytes(4)
    assert e.value.status == -3
    with pytest.raises(ValueError):
        bnn.Net().add_fc(to_dev(wl.random_bits(rng, 10, 64, 2)), None, 64)


def test_persistent_bits_input_and_limits(bnn, orc):
    rng = np.random.default_rng(3)
    dims = (200, 96, 70, 5)
    W = [wl.random_bits(rng, dims[i + 1], dims[i], wl.round_up(wl.nwords(dims[i]), 4)) for i in range(3)]
    thr = [wl.random_thresholds(rng, dims[i + 1], -8, 8) for i in range(2)]
    x = wl.random_bits(rng, 50, dims[0], wl.round_up(wl.nwords(dims[0]), 4))
    net = bnn.Net()
    net.input_bits(dims[0])
    for i in range(3):
        net.add_fc(to_dev(W[i]), to_dev(thr[i]) if i < 2 else None, dims[i])
    h = x
    for i in range(2):
        h = orc.threshold_pack(orc.bmm(h, W[i], dims[i]), thr[i], ldb_w=wl.round_up(wl.nwords(dims[i + 1]), 4))
    ref = orc.bmm(h, W[2], dims[2])
    assert np.array_equal(host(net.forward_persistent(to_dev(x))), ref)
    # a convolutional network with pooling layers: every run of layers between the pools is one persistent launch,
    # the result is that of the per-layer forward (Cifar-VGG and Cifar-ResNet-14: convolutions, blocks, then FC layers)
    for name in ("cifar_vgg", "cifar_resnet14"):
        spec = wl.cnn_layers(name)
        cnn = bnn.Net.from_layers(spec["layers"], spec["in_hw"])
        xi = to_dev(wl.cnn_input(name, 3))
        want = host(cnn.forward(xi))
        for rep in range(2):
            assert np.array_equal(host(cnn.forward_persistent(xi)), want), (name, rep)
            assert not cnn.persistent_status()


@pytest.mark.parametrize("shape", [(2, 21, 19, 3, 5, 7, 4, 3), (1, 9, 9, 1, 1, 3, 1, 1), (3, 16, 12, 4, 70, 5, 2, 2),
                                   (2, 32, 32, 3, 64, 7, 4, 3), (1, 8, 8, 2, 33, 1, 1, 0), (5, 64, 64, 3, 64, 7, 4, 3),
                                   (2, 33, 31, 3, 130, 3, 1, 1),
                                   # the kernel with wave-private patches in LDS (pixel step a multiple of 8 bytes in bf16):
                                   # ragged rectangles, pad 0 and pad > 0, several channel tiles, one-pixel outputs, a 4-channel
                                   # stride-1 layer, more images than waves
                                   (3, 37, 41, 3, 64, 7, 4, 3), (2, 30, 30, 3, 100, 7, 4, 0), (1, 7, 7, 3, 64, 7, 4, 0),
                                   (2, 19, 23, 4, 40, 3, 1, 1), (1, 5, 6, 8, 33, 3, 1, 1), (300, 9, 9, 3, 64, 5, 4, 2),
                                   (2, 48, 52, 6, 64, 3, 2, 1), (1, 224, 224, 3, 64, 7, 4, 3)])
@pytest.mark.parametrize("products", [9, 6])
def test_conv_f32_split_shapes(bnn, orc, shape, products):
    # the fp32 first layer on the bf16 matrix cores (three-way exact split of inputs and weights; all nine term
    # products, or the six that reach fp32 precision)
    N, H, W, C, O, k, st, pad = shape
    rng = np.random.default_rng(sum(shape) + 3)
    x = rng.uniform(-1, 1, size=(N, H, W, C)).astype(np.float32)
    w = rng.normal(0, 0.05, size=(O, k, k, C)).astype(np.float32)
    thr = rng.normal(0, 0.05, size=O).astype(np.float32)
    bits, y = bnn.conv_f32_split_thr(to_dev(x), to_dev(w), to_dev(thr), st, pad, want_f32=True, products=products)
    ref = orc.conv_f32(x, w, st, pad)
    tol = 1e-4 * np.maximum(np.abs(ref), np.sqrt((ref.astype(np.float64) ** 2).mean()))
    assert host(y).shape == ref.shape
    assert (np.abs(host(y) - ref) <= tol).all()
    # far tighter in fact: the products are exact (or, with six, as good as rounded to fp32), the fp32 additions round
    assert np.abs(host(y) - ref).max() <= 2e-6 * np.abs(w).max() * np.sqrt(k * k * C) * 4
    assert np.array_equal(words(bits), orc.pack_f32(host(y), thr))
    assert np.array_equal(words(bnn.conv_f32_split_thr(to_dev(x), to_dev(w), to_dev(thr), st, pad, products=products)),
                          words(bits))


def test_conv_f32_split_exact_products(bnn, orc):
    # integer inputs and weights whose products need all 24 + 24 significand bits pairwise: with every term product
    # formed, sums that stay below 2^24 are exact, so the result equals the oracle's bit for bit
    rng = np.random.default_rng(6)
    x = rng.integers(-2000, 2001, size=(2, 12, 13, 3)).astype(np.float32)
    w = rng.integers(-50, 51, size=(40, 5, 5, 3)).astype(np.float32)
    zero = to_dev(np.zeros(40, np.float32))
    _, y = bnn.conv_f32_split_thr(to_dev(x), to_dev(w), zero, 2, 2, want_f32=True)
    ref = orc.conv_f32(x, w, 2, 2)
    assert np.abs(ref).max() < 2 ** 24 and np.array_equal(host(y), ref)
    # one isolated full-precision product: (2^24 - 1) / 2^12 times (2^24 - 3) / 2^20 rounded once, as fp32 does
    x = np.zeros((1, 9, 9, 3), np.float32)
    w = np.zeros((3, 3, 3, 3), np.float32)
    x[0, 4, 4, 1] = 16777215.0 / 4096
    w[2, 1, 1, 1] = 16777213.0 / 1048576
    _, y = bnn.conv_f32_split_thr(to_dev(x), to_dev(w), to_dev(np.zeros(3, np.float32)), 1, 1, want_f32=True)
    assert host(y)[0, 4, 4, 2] == np.float32(np.float64(x[0, 4, 4, 1]) * np.float64(w[2, 1, 1, 1]))
    assert np.array_equal(host(y), orc.conv_f32(x, w, 1, 1))
