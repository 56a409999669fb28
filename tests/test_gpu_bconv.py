"""GPU parity: bnn_bconv / bnn_bconv_thr through the C ABI against the CPU oracle, bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import host, to_dev, words

pytestmark = pytest.mark.gpu

PATHS = [("valu", 1), ("mfma", 2)]


@pytest.fixture(scope="module")
def bnn():
    import paper_2006_16578_amd as b
    b.load()
    return b


def run_conv(bnn, orc, case, path, pad_mode, ref=None, with_resid=True):
    x, f, tau = to_dev(case["x"]), to_dev(case["filt"]), to_dev(case["tau"])
    C, st, pad = case["C"], case["stride"], case["pad"]
    ref = orc.bconv(case["x"], case["filt"], C, st, pad, pad_mode) if ref is None else ref
    got = host(bnn.bconv(x, f, C, st, pad, pad_mode, path=path))
    assert got.shape == ref.shape
    assert np.array_equal(got, ref), "int32 mismatch: %d wrong" % int((got != ref).sum())
    bits = words(bnn.bconv_thr(x, f, tau, C, st, pad, pad_mode, path=path))
    assert np.array_equal(bits, orc.threshold_pack(ref, case["tau"])), "bit mismatch"
    if with_resid:
        rng = np.random.default_rng(ref.size % 9973)
        R = rng.integers(-300, 301, size=ref.shape).astype(np.int32)
        bits2, S = bnn.bconv_thr(x, f, tau, C, st, pad, pad_mode, residual=to_dev(R), want_sum=True, path=path)
        assert np.array_equal(host(S), ref + R)
        assert np.array_equal(words(bits2), orc.threshold_pack(ref + R, case["tau"]))


SMALL = [  # N, H, W, C, O, k, stride, pad
    (1, 1, 1, 1, 1, 1, 1, 0), (1, 3, 3, 1, 1, 3, 1, 1), (2, 5, 4, 3, 3, 3, 1, 1), (2, 5, 4, 32, 3, 3, 2, 1),
    (2, 7, 6, 33, 5, 3, 1, 1), (3, 8, 8, 64, 40, 3, 1, 1), (2, 9, 7, 96, 33, 3, 2, 1), (2, 6, 6, 128, 64, 1, 2, 0),
    (1, 11, 10, 160, 70, 5, 2, 2), (2, 12, 12, 256, 96, 3, 1, 1), (1, 7, 7, 512, 130, 3, 1, 1),
    (5, 14, 14, 64, 128, 3, 2, 1), (3, 10, 9, 192, 65, 3, 1, 0), (2, 8, 8, 320, 32, 1, 1, 0),
    # 3x3 windows of 64 / 128 / 256 / 512 channels (the unrolled form) without padding, with pad 2, with images
    # smaller than the window, with stride 3
    (2, 9, 8, 64, 33, 3, 1, 0), (2, 9, 8, 128, 33, 3, 2, 2), (1, 2, 2, 256, 8, 3, 1, 1), (2, 11, 13, 512, 64, 3, 3, 2),
    (3, 1, 5, 128, 40, 3, 1, 1)]


@pytest.mark.parametrize("pad_mode", [0, 1])
@pytest.mark.parametrize("pname,path", PATHS)
def test_small_shapes(bnn, orc, pname, path, pad_mode):
    for idx, (N, H, W, C, O, k, st, pad) in enumerate(SMALL):
        print("conv", N, H, W, C, O, k, st, pad, pname, pad_mode, flush=True)
        case = wl.bconv_case(92, N, H, W, C, O, k, st, pad, index0=10 * idx)
        run_conv(bnn, orc, case, path, pad_mode)


# ragged shapes that select the LDS-staged convolution kernels (16-byte pixels and 8-byte pixels)
STAGED = [(5, 60, 60, 128, 130, 7, 1, 3, "mfma_fp4_conv_lds_wg128x128"),
          (8, 70, 70, 64, 100, 9, 1, 4, "mfma_fp4_conv_lds_wg128x128"),
          (9, 57, 57, 512, 300, 3, 2, 1, "mfma_fp4_conv_wg64x64"),
          (33, 40, 40, 384, 70, 5, 1, 2, "mfma_fp4_conv_lds_wg128x128"),
          (70, 58, 58, 384, 40, 5, 1, 2, "mfma_fp4_conv_lds_wg512x64"),
          (5, 60, 60, 256, 130, 7, 1, 3, "mfma_fp4_conv_lds_wg128x128"),
          (64, 64, 64, 128, 256, 7, 1, 3, "mfma_fp4_conv_lds_wg256x128")]


@pytest.mark.parametrize("shape", STAGED)
def test_ragged_shapes_staged_tiles(bnn, orc, shape):
    N, H, W, C, O, k, st, pad, kernel = shape
    assert bnn.bconv_kernel_name(N, H, W, C, O, k, st, pad) == kernel
    case = wl.bconv_case(94, N, H, W, C, O, k, st, pad, index0=C % 89)
    for pad_mode in (0, 1):
        ref1 = orc.bconv(case["x"], case["filt"], C, st, pad, pad_mode, tier=1)
        assert np.array_equal(orc.bconv_images(case["x"], case["filt"], C, st, pad, pad_mode, N - 1, 1), ref1[N - 1:])
        run_conv(bnn, orc, case, 0, pad_mode, ref=ref1)


def test_paper_sweep_shape_c640(bnn, orc):
    # one shape of the paper's BConv sweep (batch 16, 64x64, 3x3, C = O = 640), as bench.py runs it
    case = wl.bconv_case(6, 16, 64, 64, 640, 640, 3, 1, 1, index0=640 % 97)
    ref1 = orc.bconv(case["x"], case["filt"], 640, 1, 1, 0, tier=1)
    assert np.array_equal(orc.bconv_images(case["x"], case["filt"], 640, 1, 1, 0, 15, 1), ref1[15:])
    run_conv(bnn, orc, case, 0, 0, ref=ref1, with_resid=False)


def test_worked_example(bnn):
    # one +1 pixel, 3x3 filter of +1, pad 1: -7 with -1 padding, +1 with excluded taps
    x = torch.ones((1, 1, 1, 1), dtype=torch.int32, device="cuda")
    f = torch.ones((1, 3, 3, 1), dtype=torch.int32, device="cuda")
    for path in (1, 2):
        assert int(bnn.bconv(x, f, 1, 1, 1, 0, path=path).item()) == -7
        assert int(bnn.bconv(x, f, 1, 1, 1, 1, path=path).item()) == 1


@pytest.mark.parametrize("which", ["4a", "4b"])
def test_cfg4_full_size(bnn, orc, which):
    # the graded shapes at full batch: all of the output against the packed tier-1 oracle, two
    # images against the naive tier-0 oracle; both pad modes; automatic path plus both explicit ones
    case = wl.cfg4a() if which == "4a" else wl.cfg4b()
    C, st, pad = case["C"], case["stride"], case["pad"]
    for pad_mode in (0, 1):
        ref1 = orc.bconv(case["x"], case["filt"], C, st, pad, pad_mode, tier=1)
        for n0 in (0, case["N"] - 1):
            assert np.array_equal(orc.bconv_images(case["x"], case["filt"], C, st, pad, pad_mode, n0, 1), ref1[n0:n0 + 1])
        for path in (0, 1, 2):
            print("cfg", which, "pad_mode", pad_mode, "path", path, flush=True)
            run_conv(bnn, orc, case, path, pad_mode, ref=ref1, with_resid=(path == 0))


@pytest.mark.parametrize("pad_mode", [0, 1])
@pytest.mark.parametrize("pname,path", [("auto", 0)] + PATHS)
def test_threshold_edge_values(bnn, orc, pname, path, pad_mode):
    # thresholds at and beyond the range of the sums and at the ends of int32.  An all +1 image under all +1 /
    # all -1 filters makes interior sums reach +k*k*C and -k*k*C exactly, so tau = +-K decides real equalities
    imin, imax = np.iinfo(np.int32).min, np.iinfo(np.int32).max
    for (N, H, W, C, O, k, st, pad) in ((2, 9, 8, 64, 48, 3, 1, 1), (1, 12, 12, 128, 40, 3, 1, 1), (2, 7, 7, 40, 33, 3, 2, 1),
                                        (1, 6, 6, 96, 64, 1, 1, 0)):
        case = wl.bconv_case(95, N, H, W, C, O, k, st, pad, index0=C % 83)
        K = k * k * C
        ones = np.full(wl.nwords(C), 0xFFFFFFFF, dtype=np.uint32)
        if C % 32:
            ones[-1] = np.uint32((1 << (C % 32)) - 1)
        case["x"][0] = ones                                  # image 0 is all +1
        edge = [K, K + 1, -K, -K - 1, K - 1, -K + 1, imin, imax, imin + 1, imax - 1, 0, 1 << 24, -(1 << 24)]
        for j, t in enumerate(edge):
            case["tau"][j] = t
            case["tau"][O - 1 - j] = t
            case["filt"][j] = ones if j % 2 == 0 else 0
            case["filt"][O - 1 - j] = 0 if j % 2 == 0 else ones
        ref = orc.bconv(case["x"], case["filt"], C, st, pad, pad_mode)
        assert (ref == K).any() and (ref == -K).any()
        print("edge thresholds conv", N, H, W, C, O, k, st, pad, pname, pad_mode, flush=True)
        run_conv(bnn, orc, case, path, pad_mode, ref=ref)


def test_error_codes(bnn):
    x = torch.zeros((1, 4, 4, 1), dtype=torch.int32, device="cuda")
    f = torch.zeros((2, 3, 3, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(bnn.BnnError) as e:
        bnn.bconv(x, f, 32, 0, 1)                 # stride 0
    assert e.value.status == -1
    with pytest.raises(bnn.BnnError) as e:
        bnn.bconv(x, f, 32, 1, 1, pad_mode=5)
    assert e.value.status == -1
    f7 = torch.zeros((2, 7, 7, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(bnn.BnnError) as e:
        bnn.bconv(x, f7, 32, 1, 1)                # window larger than the padded image
    assert e.value.status == -1


@pytest.mark.parametrize("shape", [(2, 6, 5, 40, 3, 3, 1, 1), (3, 20, 20, 128, 64, 3, 1, 1), (2, 17, 13, 96, 70, 3, 2, 1),
                                   (1, 9, 9, 33, 5, 1, 1, 0)])
@pytest.mark.parametrize("pad_mode", [0, 1])
def test_general_bconv_f32(bnn, orc, shape, pad_mode):
    # Sec. 7.3 "general" BConv: real-valued input and filter, real-valued output
    N, H, W, C, O, k, st, pad = shape
    rng = np.random.default_rng(sum(shape) + pad_mode)
    x = rng.normal(size=(N, H, W, C)).astype(np.float32)
    f = rng.normal(size=(O, k, k, C)).astype(np.float32)
    got = host(bnn.bconv_general_f32(to_dev(x), to_dev(f), st, pad, pad_mode))
    assert got.dtype == np.float32 and np.array_equal(got, orc.general_bconv_f32(x, f, st, pad, pad_mode))


def _random_conv_shapes(seed, count):
    """Seeded random convolution shapes inside the documented limits, biased to the cases the kernels branch on:
    channel counts around multiples of 32 / 64 / 128 / 256, windows 1..7, strides 1..3, every legal padding."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        C = int(rng.choice([1, 31, 32, 33, 64, 65, 96, 128, 160, 192, 256, 257, 384, 512]))
        k = int(rng.choice([1, 2, 3, 3, 3, 4, 5, 7]))
        st = int(rng.integers(1, 4))
        pad = int(rng.integers(0, k))
        H, W = int(rng.integers(1, 15)), int(rng.integers(1, 15))
        if H + 2 * pad < k or W + 2 * pad < k or k * k * C > 20000:
            continue
        N = int(rng.integers(1, 5))
        O = int(rng.choice([1, 7, 32, 33, 64, 70, 128, 130]))
        shapes.append((N, H, W, C, O, k, st, pad))
    return shapes


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_shapes_all_paths(bnn, orc, seed):
    # 60 random shapes per seed: int32 sums, threshold -> bits, residual in and sum out, both padding conventions,
    # on the automatic choice and on both explicit paths
    for idx, (N, H, W, C, O, k, st, pad) in enumerate(_random_conv_shapes(seed, 60)):
        print("conv", N, H, W, C, O, k, st, pad, flush=True)
        case = wl.bconv_case(seed, N, H, W, C, O, k, st, pad, index0=10 * idx)
        for pad_mode in (0, 1):
            ref = orc.bconv(case["x"], case["filt"], C, st, pad, pad_mode)
            for path in (0, 1, 2):
                run_conv(bnn, orc, case, path, pad_mode, ref=ref)


# shapes large enough for each of the bigger workgroup tiles of the direct kernel (512x64, 256x128, 128x128), with
# ragged last tiles, odd channel counts, strides and paddings; residual in and sum out as well
LARGER = [(150, 61, 59, 64, 64, 3, 2, 1, "mfma_fp4_conv_wg512x64"), (41, 60, 58, 96, 40, 3, 1, 0, "mfma_fp4_conv_wg512x64"),
          (29, 61, 60, 128, 160, 3, 1, 1, "mfma_fp4_conv_wg256x128"), (50, 90, 88, 160, 130, 3, 2, 2, "mfma_fp4_conv_wg256x128"),
          (13, 59, 57, 256, 100, 3, 1, 1, "mfma_fp4_conv_wg128x128"), (11, 63, 61, 33, 128, 2, 1, 1, "mfma_fp4_conv_wg128x128")]


@pytest.mark.parametrize("shape", LARGER)
def test_larger_tiles_direct_kernel(bnn, orc, shape):
    N, H, W, C, O, k, st, pad, kernel = shape
    assert bnn.bconv_kernel_name(N, H, W, C, O, k, st, pad) == kernel
    case = wl.bconv_case(95, N, H, W, C, O, k, st, pad, index0=C % 89)
    for pad_mode in (0, 1):
        ref1 = orc.bconv(case["x"], case["filt"], C, st, pad, pad_mode, tier=1)
        assert np.array_equal(orc.bconv_images(case["x"], case["filt"], C, st, pad, pad_mode, N - 1, 1), ref1[N - 1:])
        run_conv(bnn, orc, case, 0, pad_mode, ref=ref1)


# 3x3 stride-1 pad-1 layers with at most 128 channels in and out, large enough for the kernel that keeps the filters and
# wave-private input patches in LDS: ragged last tile, ragged columns, tiles that cross image rows and whole images
# (7x7 and 1x2 images), 64 and 128 channels, an image wider than the words requested ahead
PATCH = [(64, 56, 56, 64, 64, "mfma_fp4_conv3x3_patch_wave64x64"), (4100, 7, 7, 64, 48, "mfma_fp4_conv3x3_patch_wave64x64"),
         (520, 20, 19, 128, 64, "mfma_fp4_conv3x3_patch_wave64x64"), (220, 28, 27, 128, 128, "mfma_fp4_conv3x3_patch_wave64x128"),
         (44, 62, 61, 64, 100, "mfma_fp4_conv3x3_patch_wave64x128"), (10, 250, 80, 64, 64, "mfma_fp4_conv3x3_patch_wave64x64"),
         (100000, 1, 2, 64, 40, "mfma_fp4_conv3x3_patch_wave64x64")]


# the same kernel with stride 2 (64 -> at most 128 channels, bits out): even and odd image sizes, images smaller than a
# tile, ragged columns, ragged last tile
PATCH_STRIDE2 = [(90, 56, 56, 64, 128), (760, 19, 17, 64, 128), (16500, 3, 4, 64, 100), (4200, 7, 7, 64, 128),
                 (63, 70, 60, 64, 96)]


@pytest.mark.parametrize("shape", PATCH_STRIDE2)
def test_patch_kernel_3x3_stride2(bnn, orc, shape):
    N, H, W, C, O = shape
    assert bnn.bconv_kernel_name(N, H, W, C, O, 3, 2, 1) == "mfma_fp4_conv3x3s2_patch_wave64x128"
    case = wl.bconv_case(98, N, H, W, C, O, 3, 2, 1, index0=(H * W) % 83)
    for pad_mode in (0, 1):
        print("patch stride 2", shape, "pad_mode", pad_mode, flush=True)
        ref1 = orc.bconv(case["x"], case["filt"], C, 2, 1, pad_mode, tier=1)
        for n0 in (0, N - 1):
            assert np.array_equal(orc.bconv_images(case["x"], case["filt"], C, 2, 1, pad_mode, n0, 1), ref1[n0:n0 + 1])
        run_conv(bnn, orc, case, 0, pad_mode, ref=ref1)


@pytest.mark.parametrize("shape", PATCH)
def test_patch_kernel_3x3(bnn, orc, shape):
    N, H, W, C, O, kernel = shape
    assert bnn.bconv_kernel_name(N, H, W, C, O, 3, 1, 1) == kernel
    case = wl.bconv_case(97, N, H, W, C, O, 3, 1, 1, index0=(H * W) % 83)
    for pad_mode in (0, 1):
        print("patch", shape, "pad_mode", pad_mode, flush=True)
        ref1 = orc.bconv(case["x"], case["filt"], C, 1, 1, pad_mode, tier=1)
        for n0 in (0, N - 1):
            assert np.array_equal(orc.bconv_images(case["x"], case["filt"], C, 1, 1, pad_mode, n0, 1), ref1[n0:n0 + 1])
        run_conv(bnn, orc, case, 0, pad_mode, ref=ref1)
