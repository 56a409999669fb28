"""Pins for the oracle's layer-chained forwards (CPU only): the MLP against numpy integer
matmuls, the ResNet-shaped network against torch.nn.functional.conv2d in float64."""
import numpy as np
import torch

import workloads as wl
from oracle import nets
from test_oracle_bmm import np_unpack_pm1
from test_oracle_bconv import unpack4


def test_mlp_vs_numpy(orc):
    params = wl.mlp_params()
    imgs = wl.mlp_images(8)
    scores, hidden = nets.mlp_forward(imgs, params, keep=True)
    assert scores.shape == (8, 10) and scores.dtype == np.int32
    x = np.where(imgs.astype(np.int64) >= 127, 1, -1)
    for l in range(3):
        v = x @ np_unpack_pm1(params["W"][l], params["K"][l]).T
        x = np.where(v >= params["thr"][l][None, :], 1, -1)
        assert (np_unpack_pm1(hidden[l], x.shape[1]) == x).all()
        assert (hidden[l][:, wl.nwords(x.shape[1]):] == 0).all()
    ref = x @ np_unpack_pm1(params["W"][3], params["K"][3]).T
    assert (scores == ref).all()
    assert (np.abs(scores) <= 1024).all() and (scores % 2 == 0).all()


def _torch_bconv(x_pm1, f_words, C, stride, pad):
    xt = torch.from_numpy(x_pm1.astype(np.float64)).permute(0, 3, 1, 2)
    ft = torch.from_numpy(unpack4(f_words, C).astype(np.float64)).permute(0, 3, 1, 2)
    xt = torch.nn.functional.pad(xt, (pad, pad, pad, pad), value=-1.0)
    return torch.nn.functional.conv2d(xt, ft, stride=stride).permute(0, 2, 3, 1).numpy().astype(np.int64)


def test_resnet_small_vs_torch(orc):
    # same block structure as the benchmark network, small channel counts and a 32x32 input
    blocks = ((64, 64, 1), (64, 96, 2), (96, 96, 1), (96, 128, 2))
    p = wl.resnet18_params(blocks=blocks, classes=13, config=95)
    x = wl.resnet18_input(2, hw=32, config=95)
    tr = nets.resnet18_forward(x, p, keep=True)
    # independent chain
    stem = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                      torch.from_numpy(p["stem_w"]).double().permute(0, 3, 1, 2),
                                      stride=4, padding=3).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(tr["stem_f32"], stem, rtol=1e-6, atol=1e-7)
    assert np.abs(stem).min() > 1e-6          # no stem value sits on the threshold in this case
    a = np.where(stem >= 0, 1, -1).astype(np.int64)
    assert (unpack4(tr["x0"], 64) == a).all()
    R = a.copy()
    for b, (cin, cout, st) in enumerate(blocks):
        blk = p["blocks"][b]
        v1 = _torch_bconv(a, blk["W1"], cin, st, 1)
        h = np.where(v1 >= blk["thr1"], 1, -1)
        v2 = _torch_bconv(h, blk["W2"], cout, 1, 1)
        sc = _torch_bconv(a, blk["Wd"], cin, st, 0) if "Wd" in blk else R
        S = v2 + sc
        assert (tr["S%d" % b] == S).all()
        a = np.where(S >= blk["thr2"], 1, -1)
        assert (unpack4(tr["y%d" % b], cout) == a).all()
        R = S
    pooled = a.sum(axis=(1, 2))
    assert (tr["pooled"] == pooled).all()
    hw = a.shape[1] * a.shape[2]
    logits = (pooled.astype(np.float64) / hw) @ p["fc_w"].astype(np.float64).T
    np.testing.assert_allclose(tr["logits"], logits, rtol=1e-5, atol=1e-6)
    # tier 1 gives the same bits and sums
    tr1 = nets.resnet18_forward(x, p, keep=True, tier=1)
    for key in tr:
        assert np.array_equal(tr[key], tr1[key]), key
    # injected stem bits are honoured
    x0 = tr["x0"].copy()
    x0[0, 0, 0, 0] ^= np.uint32(1)
    tr2 = nets.resnet18_forward(x, p, stem_bits=x0, keep=True)
    assert not np.array_equal(tr2["S0"], tr["S0"])


def test_cnn_forward_vgg_like_vs_torch(orc):
    # conv_f32 -> bconv -> pool -> bconv -> pool -> fc -> fc against an independent torch / numpy chain
    rng = np.random.default_rng(31)
    L = [{"op": "conv_f32", "w": rng.normal(0, 0.05, size=(64, 3, 3, 3)).astype(np.float32),
          "thr": np.zeros(64, np.float32), "stride": 1, "pad": 1},
         {"op": "bconv", "W": wl.random_bits(rng, (64, 3, 3), 64), "thr": wl.random_thresholds(rng, 64, -30, 30), "C": 64, "stride": 1, "pad": 1},
         {"op": "pool", "win": 2, "stride": 2},
         {"op": "bconv", "W": wl.random_bits(rng, (96, 3, 3), 64), "thr": wl.random_thresholds(rng, 96, -30, 30), "C": 64, "stride": 1, "pad": 1},
         {"op": "pool", "win": 2, "stride": 2},
         {"op": "fc", "W": wl.random_bits(rng, 40, 2 * 2 * 96, 12), "thr": wl.random_thresholds(rng, 40, -10, 10), "K": 2 * 2 * 96},
         {"op": "fc", "W": wl.random_bits(rng, 7, 40, 4), "thr": None, "K": 40}]
    x = rng.uniform(-1, 1, size=(3, 8, 8, 3)).astype(np.float32)
    outs = nets.cnn_forward(x, L, keep=True)
    stem = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                      torch.from_numpy(L[0]["w"]).double().permute(0, 3, 1, 2), padding=1).permute(0, 2, 3, 1).numpy()
    assert np.abs(stem).min() > 1e-6
    a = np.where(stem >= 0, 1, -1).astype(np.int64)
    assert (unpack4(outs[0], 64) == a).all()
    a = np.where(_torch_bconv(a, L[1]["W"], 64, 1, 1) >= L[1]["thr"], 1, -1)
    assert (unpack4(outs[1], 64) == a).all()
    a = a.reshape(3, 4, 2, 4, 2, 64).max(axis=(2, 4))
    assert (unpack4(outs[2], 64) == a).all()
    a = np.where(_torch_bconv(a, L[3]["W"], 64, 1, 1) >= L[3]["thr"], 1, -1)
    a = a.reshape(3, 2, 2, 2, 2, 96).max(axis=(2, 4))
    assert (unpack4(outs[4], 96) == a).all()
    flat = a.reshape(3, -1)                                           # NHWC flatten
    v = flat @ np_unpack_pm1(L[5]["W"], 384).T
    a = np.where(v >= L[5]["thr"], 1, -1)
    assert (np_unpack_pm1(outs[5], 40) == a).all() and (outs[5][:, 2:] == 0).all()
    assert (outs[6] == a @ np_unpack_pm1(L[6]["W"], 40).T).all()


def _torch_conv_pm1(x_pm1, f_words, C, stride, pad, pad_value):
    """Independent +1/-1 convolution: torch float64 conv2d over an input explicitly padded with `pad_value`
    (-1: out-of-frame inputs count as -1; 0: out-of-frame taps contribute nothing)."""
    xt = torch.from_numpy(x_pm1.astype(np.float64)).permute(0, 3, 1, 2)
    ft = torch.from_numpy(unpack4(f_words, C).astype(np.float64)).permute(0, 3, 1, 2)
    xt = torch.nn.functional.pad(xt, (pad, pad, pad, pad), value=float(pad_value))
    return torch.nn.functional.conv2d(xt, ft, stride=stride).permute(0, 2, 3, 1).numpy().astype(np.int64)


def test_resnet_exclude_padding_vs_torch(orc):
    # the paper's padding convention (Sec. 5.3: out-of-frame taps are excluded) through the whole residual
    # chain: every convolution of every block against torch on an input padded with ZEROS.  Forgetting the
    # pad mode on any one of the three convolutions of a block changes the border sums of that block.
    blocks = ((64, 64, 1), (64, 96, 2), (96, 96, 1), (96, 128, 2))
    p = wl.resnet18_params(blocks=blocks, classes=13, config=97)
    x = wl.resnet18_input(2, hw=32, config=97)
    tr = nets.resnet18_forward(x, p, keep=True, pad_mode=orc.PAD_EXCLUDE)
    tr_m1 = nets.resnet18_forward(x, p, keep=True)
    stem = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                      torch.from_numpy(p["stem_w"]).double().permute(0, 3, 1, 2),
                                      stride=4, padding=3).permute(0, 2, 3, 1).numpy()
    assert np.abs(stem).min() > 1e-6
    a = np.where(stem >= 0, 1, -1).astype(np.int64)
    R = a.copy()
    differs_from_minus_one = 0
    for b, (cin, cout, st) in enumerate(blocks):
        blk = p["blocks"][b]
        v1 = _torch_conv_pm1(a, blk["W1"], cin, st, 1, 0)
        h = np.where(v1 >= blk["thr1"], 1, -1)
        assert (unpack4(tr["h%d" % b], cout) == h).all(), "block %d hidden bits" % b
        v2 = _torch_conv_pm1(h, blk["W2"], cout, 1, 1, 0)
        sc = _torch_conv_pm1(a, blk["Wd"], cin, st, 0, 0) if "Wd" in blk else R
        S = v2 + sc
        assert (tr["S%d" % b] == S).all(), "block %d sums" % b
        a = np.where(S >= blk["thr2"], 1, -1)
        assert (unpack4(tr["y%d" % b], cout) == a).all()
        R = S
        differs_from_minus_one += int((tr["S%d" % b] != tr_m1["S%d" % b]).sum())
    assert differs_from_minus_one > 0                  # the two conventions are really different on this case
    assert (tr["pooled"] == a.sum(axis=(1, 2))).all()
    tr1 = nets.resnet18_forward(x, p, keep=True, tier=1, pad_mode=orc.PAD_EXCLUDE)
    for key in tr:
        assert np.array_equal(tr[key], tr1[key]), key


def test_cnn_forward_bwn_and_blocks_vs_torch(orc):
    # bwn first layer -> bconv -> identity block (residual starts from the bits) -> block with a 1x1 shortcut
    # -> identity block (residual is the previous block's sum) -> fc, against an independent torch / numpy chain
    rng = np.random.default_rng(77)

    def block(cin, cout, stride):
        b = {"op": "block", "cin": cin, "cout": cout, "stride": stride,
             "W1": wl.random_bits(rng, (cout, 3, 3), cin), "thr1": wl.random_thresholds(rng, cout, -30, 30),
             "W2": wl.random_bits(rng, (cout, 3, 3), cout), "thr2": wl.random_thresholds(rng, cout, -30, 30)}
        if stride != 1 or cin != cout:
            b["Wd"] = wl.random_bits(rng, (cout, 1, 1), cin)
        return b

    L = [{"op": "bwn", "W": wl.random_bits(rng, (40, 3, 3), 3), "thr": rng.normal(0, 0.3, size=40).astype(np.float32),
          "C": 3, "stride": 1, "pad": 1},
         {"op": "bconv", "W": wl.random_bits(rng, (64, 3, 3), 40), "thr": wl.random_thresholds(rng, 64, -30, 30),
          "C": 40, "stride": 1, "pad": 1},
         block(64, 64, 1), block(64, 96, 2), block(96, 96, 1),
         {"op": "fc", "W": wl.random_bits(rng, 9, 5 * 5 * 96, wl.round_up(wl.nwords(5 * 5 * 96), 4)), "thr": None,
          "K": 5 * 5 * 96}]
    x = rng.uniform(-1, 1, size=(2, 10, 10, 3)).astype(np.float32)
    outs = nets.cnn_forward(x, L, keep=True)
    # first layer: weight bit 1 adds the input element, bit 0 subtracts it; zero padding; fp32 threshold
    w_pm1 = torch.from_numpy(unpack4(L[0]["W"], 3).astype(np.float64)).permute(0, 3, 1, 2)
    y0 = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2), w_pm1, padding=1)
    y0 = y0.permute(0, 2, 3, 1).numpy()
    assert np.abs(y0 - L[0]["thr"]).min() > 1e-5          # no value sits on its threshold in this case
    a = np.where(y0 >= L[0]["thr"].astype(np.float64), 1, -1).astype(np.int64)
    assert (unpack4(outs[0], 40) == a).all()
    assert (outs[0][..., 1] >> 8 == 0).all()              # pad bits of the 40-channel pixel are zero
    a = np.where(_torch_conv_pm1(a, L[1]["W"], 40, 1, 1, -1) >= L[1]["thr"], 1, -1)
    assert (unpack4(outs[1], 64) == a).all()
    R = a.copy()                                          # first block of the chain: residual = +1/-1 of its input
    for i in (2, 3, 4):
        B = L[i]
        v1 = _torch_conv_pm1(a, B["W1"], B["cin"], B["stride"], 1, -1)
        h = np.where(v1 >= B["thr1"], 1, -1)
        v2 = _torch_conv_pm1(h, B["W2"], B["cout"], 1, 1, -1)
        sc = _torch_conv_pm1(a, B["Wd"], B["cin"], B["stride"], 0, -1) if "Wd" in B else R
        S = v2 + sc
        a = np.where(S >= B["thr2"], 1, -1)
        assert (unpack4(outs[i], B["cout"]) == a).all(), "block layer %d" % i
        R = S
    assert (outs[5] == a.reshape(2, -1) @ np_unpack_pm1(L[5]["W"], 5 * 5 * 96).T).all()
    # the residual entering the last block really is the previous sum, not +-1: dropping it changes the bits
    Lmut = [dict(l) for l in L]
    Lmut[4] = dict(L[4]); Lmut[4]["Wd"] = wl.random_bits(rng, (96, 1, 1), 96)
    assert not np.array_equal(nets.cnn_forward(x, Lmut, keep=True)[4], outs[4])
