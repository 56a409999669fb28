"""Pins for the oracle's bit convolution and the fp32 end layers (CPU only).

Independent formulations used here: (a) an explicitly padded +1/-1/0 image followed by a *valid*
cross-correlation written with numpy slicing, (b) torch.nn.functional.conv2d in float64 on CPU
(exact: all partial sums are small integers), (c) closed forms for all-ones operands, (d) the
worked examples in tests/golden/worked_examples.txt, (e) 1x1 convolution == BMM.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from test_oracle_bmm import golden, np_unpack_pm1


def unpack4(words, C):
    shp = words.shape[:-1]
    return np_unpack_pm1(words.reshape(-1, words.shape[-1]), C).reshape(shp + (C,))


def conv_by_padding(x_pm1, f_pm1, stride, pad, pad_value):
    """x [N][H][W][C], f [O][k][k][C] int -> [N][P][Q][O]; materialise the padded image."""
    N, H, W, C = x_pm1.shape
    O, k, _, _ = f_pm1.shape
    xp = np.full((N, H + 2 * pad, W + 2 * pad, C), pad_value, dtype=np.int64)
    xp[:, pad:pad + H, pad:pad + W, :] = x_pm1
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    out = np.zeros((N, P, Q, O), dtype=np.int64)
    for r in range(k):
        for s in range(k):
            win = xp[:, r:r + (P - 1) * stride + 1:stride, s:s + (Q - 1) * stride + 1:stride, :]
            out += np.einsum("npqc,oc->npqo", win, f_pm1[:, r, s, :].astype(np.int64))
    return out


def test_golden_conv(orc):
    x = np.array([[[[1]]]], dtype=np.uint32)
    f = np.full((1, 3, 3, 1), 1, dtype=np.uint32)
    for args, exp in golden("conv"):
        assert orc.bconv(x, f, 1, 1, 1, int(args["pad_mode"]))[0, 0, 0, 0] == exp
        assert orc.bconv(x, f, 1, 1, 1, int(args["pad_mode"]), tier=1)[0, 0, 0, 0] == exp


CASES = [(N, H, W, C, O, k, st, pad)
         for (N, H, W) in ((1, 3, 3), (2, 5, 4))
         for C in (1, 3, 32, 33, 64)
         for O in (1, 3)
         for (k, st, pad) in ((1, 1, 0), (1, 2, 0), (3, 1, 1), (3, 2, 1), (3, 1, 0), (3, 2, 0))]


@pytest.mark.parametrize("pad_mode", [0, 1])
def test_small_vs_padded_formulation(orc, pad_mode):
    rng = np.random.default_rng(42 + pad_mode)
    for (N, H, W, C, O, k, st, pad) in CASES:
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        x = wl.random_bits(rng, (N, H, W), C)
        f = wl.random_bits(rng, (O, k, k), C)
        ref = conv_by_padding(unpack4(x, C), unpack4(f, C), st, pad, -1 if pad_mode == 0 else 0)
        got = orc.bconv(x, f, C, st, pad, pad_mode)
        assert got.shape == ref.shape
        assert (got == ref).all(), (N, H, W, C, O, k, st, pad)
        assert (orc.bconv(x, f, C, st, pad, pad_mode, tier=1) == ref).all()


@pytest.mark.parametrize("pad_mode", [0, 1])
@pytest.mark.parametrize("shape", [(2, 9, 7, 64, 5, 3, 1, 1), (3, 8, 8, 96, 4, 3, 2, 1), (2, 6, 6, 40, 7, 1, 2, 0),
                                   (1, 11, 10, 128, 3, 5, 2, 2)])
def test_vs_torch_conv2d(orc, shape, pad_mode):
    N, H, W, C, O, k, st, pad = shape
    rng = np.random.default_rng(sum(shape))
    x = wl.random_bits(rng, (N, H, W), C)
    f = wl.random_bits(rng, (O, k, k), C)
    xt = torch.from_numpy(unpack4(x, C).astype(np.float64)).permute(0, 3, 1, 2)     # NCHW
    ft = torch.from_numpy(unpack4(f, C).astype(np.float64)).permute(0, 3, 1, 2)     # OCkk
    xt = torch.nn.functional.pad(xt, (pad, pad, pad, pad), value=-1.0 if pad_mode == 0 else 0.0)
    ref = torch.nn.functional.conv2d(xt, ft, stride=st, padding=0).permute(0, 2, 3, 1).numpy()
    got = orc.bconv(x, f, C, st, pad, pad_mode)
    assert (got == ref.astype(np.int64)).all()
    assert (orc.bconv(x, f, C, st, pad, pad_mode, tier=1) == got).all()
    assert (orc.bconv_images(x, f, C, st, pad, pad_mode, N - 1, 1) == got[N - 1:]).all()


def test_closed_form_all_ones(orc):
    # all +1 image and filter, k = 3, pad = 1, stride 1: valid taps are 4 (corner), 6 (edge), 9
    C, H, W = 40, 5, 6
    x = np.zeros((1, H, W, 2), np.uint32)
    x[..., 0] = 0xFFFFFFFF
    x[..., 1] = 0xFF
    f = np.zeros((2, 3, 3, 2), np.uint32)
    f[..., 0] = 0xFFFFFFFF
    f[..., 1] = 0xFF
    valid = np.full((H, W), 9)
    valid[0, :] = valid[-1, :] = 6
    valid[:, 0] = valid[:, -1] = 6
    valid[0, 0] = valid[0, -1] = valid[-1, 0] = valid[-1, -1] = 4
    m1 = orc.bconv(x, f, C, 1, 1, 0)
    ex = orc.bconv(x, f, C, 1, 1, 1)
    for o in range(2):
        assert (m1[0, :, :, o] == C * (2 * valid - 9)).all()
        assert (ex[0, :, :, o] == C * valid).all()


def test_invariants(orc):
    rng = np.random.default_rng(8)
    N, H, W, C, O, k = 2, 6, 6, 70, 4, 3
    x = wl.random_bits(rng, (N, H, W), C)
    f = wl.random_bits(rng, (O, k, k), C)
    m1 = orc.bconv(x, f, C, 1, 1, 0)
    ex = orc.bconv(x, f, C, 1, 1, 1)
    # parity and bound with the full window in -1 mode
    assert ((m1 - C * 9) % 2 == 0).all() and (np.abs(m1) <= C * 9).all()
    # interior pixels are identical in both modes; borders differ by the sum of the filter taps
    # that fall outside (a per-border-class constant): check one corner explicitly
    assert (m1[:, 1:-1, 1:-1] == ex[:, 1:-1, 1:-1]).all()
    fp = unpack4(f, C)
    outside = fp[:, 0, :, :].sum(axis=(1, 2)) + fp[:, 1:, 0, :].sum(axis=(1, 2))   # taps r=0 or s=0
    assert (ex[:, 0, 0, :] - m1[:, 0, 0, :] == outside[None, :]).all()
    # 1x1 stride-1 convolution is a BMM over the [N*H*W][C] matrix
    f1 = wl.random_bits(rng, (O, 1, 1), C)
    c1 = orc.bconv(x, f1, C, 1, 0, 0)
    mm = orc.bmm(x.reshape(-1, x.shape[-1]), f1.reshape(O, -1), C)
    assert (c1.reshape(-1, O) == mm).all()
    # flipping one input bit moves every affected output by exactly 2
    x2 = x.copy()
    x2[1, 3, 2, 1] ^= np.uint32(1 << 5)
    d = orc.bconv(x2, f, C, 1, 1, 0) - m1
    assert set(np.unique(np.abs(d))) <= {0, 2}
    assert (np.abs(d[1, 2:5, 1:4]) == 2).all() and (d[0] == 0).all()


def test_cfg4_slab_tiers_agree(orc):
    # the two graded conv shapes on two images: tier 0 == tier 1, statistics as expected
    for case in (wl.cfg4a(2), wl.cfg4b(2)):
        a = orc.bconv(case["x"], case["filt"], case["C"], case["stride"], case["pad"], 0)
        b = orc.bconv(case["x"], case["filt"], case["C"], case["stride"], case["pad"], 0, tier=1)
        assert (a == b).all()
        Kt = 9 * case["C"]
        assert abs(a[:, 1:-1, 1:-1].var() / Kt - 1.0) < 0.05


def test_conv_f32_vs_torch(orc):
    rng = np.random.default_rng(2)
    x = rng.uniform(-1, 1, size=(2, 21, 19, 3)).astype(np.float32)
    w = rng.normal(0, 0.02, size=(5, 7, 7, 3)).astype(np.float32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                     torch.from_numpy(w).double().permute(0, 3, 1, 2),
                                     stride=4, padding=3).permute(0, 2, 3, 1).numpy()
    got = orc.conv_f32(x, w, 4, 3)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-7)


def test_sumpool_and_head(orc):
    rng = np.random.default_rng(4)
    C = 70
    bits = wl.random_bits(rng, (3, 7, 7), C)
    pooled = orc.sumpool_pm1(bits, C)
    ref = unpack4(bits, C).sum(axis=(1, 2))
    assert (pooled == ref).all() and (np.abs(pooled) <= 49).all() and ((pooled - 49) % 2 == 0).all()
    w = rng.normal(0, 0.02, size=(11, C)).astype(np.float32)
    y = orc.head_fc_f32(pooled, w, 49.0)
    yref = (pooled.astype(np.float64) / 49.0) @ w.astype(np.float64).T
    np.testing.assert_allclose(y, yref, rtol=1e-5, atol=1e-7)


def test_maxpool_vs_torch_and_closed_forms(orc):
    rng = np.random.default_rng(21)
    for (N, H, W, C, win, st) in [(2, 8, 8, 40, 2, 2), (1, 7, 9, 64, 2, 2), (3, 6, 6, 33, 3, 1), (1, 5, 5, 1, 2, 1)]:
        bits = wl.random_bits(rng, (N, H, W), C)
        got = orc.maxpool_pm1(bits, C, win, st)
        v = torch.from_numpy(unpack4(bits, C).astype(np.float64)).permute(0, 3, 1, 2)
        ref = torch.nn.functional.max_pool2d(v, win, st).permute(0, 2, 3, 1).numpy()
        assert unpack4(got, C).shape == ref.shape
        assert (unpack4(got, C) == ref).all()
        assert (unpack4(got, wl.nwords(C) * 32)[..., C:] < 0).all()          # pad bits stay 0
    # all -1 stays -1; a single +1 anywhere in a window makes that window +1
    z = np.zeros((1, 4, 4, 1), np.uint32)
    assert (orc.maxpool_pm1(z, 32, 2, 2) == 0).all()
    z[0, 3, 2, 0] = 1 << 7
    o = orc.maxpool_pm1(z, 32, 2, 2)
    assert o[0, 1, 1, 0] == 1 << 7 and o.sum() == 1 << 7


def test_bwn_first_layer_vs_torch_and_closed_forms(orc):
    rng = np.random.default_rng(77)
    for (N, H, W, C, O, k, st, pad) in [(2, 21, 19, 3, 5, 7, 4, 3), (1, 9, 8, 3, 40, 3, 1, 1), (2, 23, 23, 3, 7, 11, 4, 2),
                                        (1, 6, 6, 35, 3, 3, 2, 1), (1, 5, 5, 1, 2, 1, 1, 0)]:
        x = rng.uniform(-1, 1, size=(N, H, W, C)).astype(np.float32)
        wb = wl.random_bits(rng, (O, k, k), C)
        ref = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                         torch.from_numpy(unpack4(wb, C).astype(np.float64)).permute(0, 3, 1, 2),
                                         stride=st, padding=pad).permute(0, 2, 3, 1).numpy()
        got = orc.bwn_conv_f32(x, wb, C, st, pad)
        assert got.shape == ref.shape
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-6)
        # same numbers as the real-valued convolution with the weights written out as +1.0 / -1.0
        np.testing.assert_allclose(got, orc.conv_f32(x, unpack4(wb, C).astype(np.float32), st, pad), rtol=1e-6, atol=1e-6)
    # all-ones weight bits: a box sum over the in-frame window; all-zero bits: its negation
    x = rng.uniform(-1, 1, size=(1, 6, 7, 3)).astype(np.float32)
    ones = np.full((1, 3, 3, 1), 0b111, np.uint32)
    xp = np.zeros((8, 9, 3))
    xp[1:-1, 1:-1] = x[0]
    box = sum(xp[r:r + 6, s:s + 7].sum(axis=2) for r in range(3) for s in range(3))
    np.testing.assert_allclose(orc.bwn_conv_f32(x, ones, 3, 1, 1)[0, :, :, 0], box, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(orc.bwn_conv_f32(x, np.zeros_like(ones), 3, 1, 1)[0, :, :, 0], -box, rtol=1e-6, atol=1e-6)


def test_general_forms_vs_numpy_sign(orc):
    rng = np.random.default_rng(78)
    A = rng.normal(size=(9, 70)).astype(np.float32)
    B = rng.normal(size=(5, 70)).astype(np.float32)
    A[0, 0] = 0.0                                         # Eq. 1: zero binarizes to +1
    B[1, 3] = -0.0
    sa, sb = np.where(A >= 0, 1, -1), np.where(B >= 0, 1, -1)
    got = orc.general_bmm_f32(A, B)
    assert got.dtype == np.float32 and (got == sa @ sb.T).all()
    x = rng.normal(size=(2, 6, 5, 40)).astype(np.float32)
    f = rng.normal(size=(3, 3, 3, 40)).astype(np.float32)
    for pm, pv in ((0, -1), (1, 0)):
        ref = conv_by_padding(np.where(x >= 0, 1, -1), np.where(f >= 0, 1, -1), 1, 1, pv)
        assert (orc.general_bconv_f32(x, f, 1, 1, pm) == ref).all()
