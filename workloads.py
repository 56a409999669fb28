"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and lays them out; it contains none of the method's
arithmetic (no dot products, no thresholds applied, no convolution).  It is the one module the
GPU tests, ``bench.py`` and the CPU oracle's tests all share.

Recipe: ``numpy.random.Generator(PCG64(seed))`` with ``seed = 20061657 + 1000 * config + index``
(index numbers the tensors of a configuration in order of use).  A packed +1/-1 operand is drawn
directly as uniform 32-bit words, which makes every bit an independent fair coin (p = 0.5); the
bits beyond the logical width are cleared, because the packed layout requires pad bits to be 0.
Thresholds are ``integers(lo, hi + 1)`` as int32.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 20061657


def seed_for(config: int, index: int) -> int:
    return SEED_BASE + 1000 * config + index


def _rng(config: int, index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed_for(config, index)))


def nwords(nbits: int) -> int:
    return (int(nbits) + 31) // 32


def round_up(v: int, m: int) -> int:
    return (int(v) + m - 1) // m * m


def random_bits(rng: np.random.Generator, shape_rows, nbits: int, ldw: int | None = None) -> np.ndarray:
    """Uniform random packed bits: array of shape (*shape_rows, ldw) uint32, pad bits zero."""
    if isinstance(shape_rows, int):
        shape_rows = (shape_rows,)
    kw = nwords(nbits)
    ldw = kw if ldw is None else ldw
    assert ldw >= kw
    w = rng.integers(0, 1 << 32, size=tuple(shape_rows) + (ldw,), dtype=np.uint64).astype(np.uint32)
    if nbits % 32:
        w[..., kw - 1] &= np.uint32((1 << (nbits % 32)) - 1)
    w[..., kw:] = 0
    return w


def random_thresholds(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    return rng.integers(lo, hi + 1, size=n, dtype=np.int64).astype(np.int32)


# ------------------------------------------------------------------------------------ config 1, 2
def bmm_case(config: int, M: int, N: int, K: int, thr_div: int = 8, index0: int = 0) -> dict:
    """A [M][ldw], B [N][ldw] random bits; tau [N] uniform integers in [-K/thr_div, K/thr_div]."""
    ldw = round_up(nwords(K), 4)
    A = random_bits(_rng(config, index0 + 0), M, K, ldw)
    B = random_bits(_rng(config, index0 + 1), N, K, ldw)
    t = K // thr_div
    tau = random_thresholds(_rng(config, index0 + 2), N, -t, t)
    return {"A": A, "B": B, "tau": tau, "M": M, "N": N, "K": K, "ldw": ldw}


CFG2_SQUARES = (2048, 4096, 8192, 16384)
CFG2_FC = ((8, 4096, 4096), (128, 4096, 4096), (1024, 4096, 4096))   # (M, N, K)


def cfg1() -> dict:
    return bmm_case(1, 1024, 1024, 1024)


def cfg2_shapes():
    """(name, M, N, K, index0) for every shape of the BMM sweep."""
    out = []
    for i, n in enumerate(CFG2_SQUARES):
        out.append(("sq%d" % n, n, n, n, 10 * i))
    for i, (m, n, k) in enumerate(CFG2_FC):
        out.append(("fc%d" % m, m, n, k, 100 + 10 * i))
    return out


def cfg2_case(name: str) -> dict:
    for nm, M, N, K, idx in cfg2_shapes():
        if nm == name:
            return bmm_case(2, M, N, K, index0=idx)
    raise KeyError(name)


# ------------------------------------------------------------------------------------ config 3
MLP_DIMS = (784, 1024, 1024, 1024, 10)


def mlp_params(dims=MLP_DIMS, config: int = 3) -> dict:
    """Random +1/-1 weights W_l [N_l][ldw_l] and per-neuron thresholds uniform in [-32, 32]."""
    W, K, thr = [], [], []
    for l in range(len(dims) - 1):
        k, n = dims[l], dims[l + 1]
        W.append(random_bits(_rng(config, 10 + l), n, k, round_up(nwords(k), 4)))
        K.append(k)
        if l < len(dims) - 2:
            thr.append(random_thresholds(_rng(config, 20 + l), n, -32, 32))
    return {"W": W, "K": K, "thr": thr, "in_thr": 127, "dims": tuple(dims)}


def mlp_images(batch: int, pixels: int = 784, config: int = 3) -> np.ndarray:
    """Synthetic 8-bit images, every pixel uniform in [0, 255]; stands in for MNIST digits."""
    return _rng(config, 0).integers(0, 256, size=(batch, pixels), dtype=np.int64).astype(np.uint8)


# ------------------------------------------------------------------------------------ config 4
def bconv_case(config: int, N: int, H: int, W: int, C: int, O: int, k: int, stride: int, pad: int,
               thr_range: int = 64, index0: int = 0) -> dict:
    x = random_bits(_rng(config, index0 + 0), (N, H, W), C)
    f = random_bits(_rng(config, index0 + 1), (O, k, k), C)
    tau = random_thresholds(_rng(config, index0 + 2), O, -thr_range, thr_range)
    return {"x": x, "filt": f, "tau": tau, "N": N, "H": H, "W": W, "C": C, "O": O, "k": k,
            "stride": stride, "pad": pad}


def cfg4a(N: int = 128) -> dict:
    return bconv_case(4, N, 56, 56, 128, 128, 3, 1, 1, index0=0)


def cfg4b(N: int = 128) -> dict:
    return bconv_case(4, N, 56, 56, 64, 128, 3, 2, 1, index0=10)


# ------------------------------------------------------------------------------------ config 5
RESNET18_BLOCKS = ((64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 128, 1),
                   (128, 256, 2), (256, 256, 1), (256, 512, 2), (512, 512, 1))


def resnet18_params(blocks=RESNET18_BLOCKS, classes: int = 1000, config: int = 5) -> dict:
    """fp32 stem [64][7][7][3] and FC [classes][512] ~ N(0, 0.02); binarized 3x3 / 1x1 weights
    random bits; thresholds uniform integers in [-64, 64]; stem threshold 0."""
    c0 = blocks[0][0]
    p = {"stem_w": _rng(config, 1).normal(0.0, 0.02, size=(c0, 7, 7, 3)).astype(np.float32),
         "stem_thr": np.zeros(c0, dtype=np.float32),
         "blocks": []}
    for b, (cin, cout, stride) in enumerate(blocks):
        blk = {"cin": cin, "cout": cout, "stride": stride,
               "W1": random_bits(_rng(config, 100 + 10 * b + 0), (cout, 3, 3), cin),
               "thr1": random_thresholds(_rng(config, 100 + 10 * b + 1), cout, -64, 64),
               "W2": random_bits(_rng(config, 100 + 10 * b + 2), (cout, 3, 3), cout),
               "thr2": random_thresholds(_rng(config, 100 + 10 * b + 3), cout, -64, 64)}
        if stride != 1 or cin != cout:
            blk["Wd"] = random_bits(_rng(config, 100 + 10 * b + 4), (cout, 1, 1), cin)
        p["blocks"].append(blk)
    p["fc_w"] = _rng(config, 2).normal(0.0, 0.02, size=(classes, blocks[-1][1])).astype(np.float32)
    return p


def resnet18_input(batch: int, hw: int = 224, config: int = 5) -> np.ndarray:
    """Synthetic images [batch][hw][hw][3] fp32 uniform in [-1, 1]; stands in for ImageNet crops."""
    return _rng(config, 0).uniform(-1.0, 1.0, size=(batch, hw, hw, 3)).astype(np.float32)


# ------------------------------------------------------------------------------------ Table-5 networks
def _conv_f32_layer(rng_w, cin, cout, k, stride, pad, scale=0.05):
    return {"op": "conv_f32", "w": rng_w.normal(0.0, scale, size=(cout, k, k, cin)).astype(np.float32),
            "thr": np.zeros(cout, dtype=np.float32), "stride": stride, "pad": pad}


def _bwn_layer(rng_w, cin, cout, k, stride, pad):
    return {"op": "bwn", "W": random_bits(rng_w, (cout, k, k), cin), "thr": np.zeros(cout, dtype=np.float32),
            "C": cin, "stride": stride, "pad": pad}


def cnn_layers(name: str, config: int = 7, first: str = "bwn") -> dict:
    """Layer lists with the shapes of the paper's Table 5 (Cifar-10 VGG and ResNet-14, ImageNet AlexNet
    and VGG-16); random +1/-1 weights, conv thresholds uniform integers in [-64, 64], FC thresholds in
    [-32, 32].  First layer (threshold 0): ``first="bwn"`` -- real-valued input, binarized weights, as the paper
    runs it (Sec. 6.1); ``first="f32"`` -- real-valued weights ~ N(0, 0.05).  "k x nFC" is read as k - 1 hidden layers of n
    neurons followed by the output layer, as the benchmark configuration reads the MLP.
    Returns {"layers", "in_hw", "classes"}."""
    idx = [0]

    def rng():
        idx[0] += 1
        return _rng(config, {"cifar_vgg": 100, "cifar_resnet14": 300, "alexnet": 500, "vgg16": 700}[name] + idx[0])

    def bconv(cin, cout, k=3, stride=1, pad=1):
        return {"op": "bconv", "W": random_bits(rng(), (cout, k, k), cin), "thr": random_thresholds(rng(), cout, -64, 64),
                "C": cin, "stride": stride, "pad": pad}

    def pool():
        return {"op": "pool", "win": 2, "stride": 2}

    def fc(k, n, last=False):
        return {"op": "fc", "W": random_bits(rng(), n, k, round_up(nwords(k), 4)),
                "thr": None if last else random_thresholds(rng(), n, -32, 32), "K": k}

    def block(cin, cout, stride):
        b = {"op": "block", "cin": cin, "cout": cout, "stride": stride,
             "W1": random_bits(rng(), (cout, 3, 3), cin), "thr1": random_thresholds(rng(), cout, -64, 64),
             "W2": random_bits(rng(), (cout, 3, 3), cout), "thr2": random_thresholds(rng(), cout, -64, 64)}
        if stride != 1 or cin != cout:
            b["Wd"] = random_bits(rng(), (cout, 1, 1), cin)
        return b

    def first_layer(cin, cout, k, stride, pad, scale=0.05):
        if first == "bwn":
            return _bwn_layer(rng(), cin, cout, k, stride, pad)
        return _conv_f32_layer(rng(), cin, cout, k, stride, pad, scale)

    if name == "cifar_vgg":          # (2x128C3)-MP2-(2x256C3)-MP2-(2x512C3)-MP2-(3x1024FC), 32x32x3 -> 10
        L = [first_layer(3, 128, 3, 1, 1), bconv(128, 128), pool(), bconv(128, 256), bconv(256, 256), pool(),
             bconv(256, 512), bconv(512, 512), pool(), fc(4 * 4 * 512, 1024), fc(1024, 1024), fc(1024, 10, last=True)]
        return {"layers": L, "in_hw": 32, "classes": 10}
    if name == "cifar_resnet14":     # 128C3/2-4x128C3-4x256C3-4x512C3-(2x512FC), 32x32x3 -> 10
        L = [first_layer(3, 128, 3, 2, 1), block(128, 128, 1), block(128, 128, 1), block(128, 256, 2),
             block(256, 256, 1), block(256, 512, 2), block(512, 512, 1), fc(4 * 4 * 512, 512), fc(512, 10, last=True)]
        return {"layers": L, "in_hw": 32, "classes": 10}
    if name == "alexnet":            # (128C11/4)-P2-(256C5)-P2-(3x256C3)-P2-(3x4096FC), 224x224x3 -> 1000
        L = [first_layer(3, 128, 11, 4, 2, scale=0.02), pool(), bconv(128, 256, 5, 1, 2), pool(),
             bconv(256, 256), bconv(256, 256), bconv(256, 256), pool(),
             fc(6 * 6 * 256, 4096), fc(4096, 4096), fc(4096, 1000, last=True)]
        return {"layers": L, "in_hw": 224, "classes": 1000}
    if name == "vgg16":              # (2x64C3)-P2-(2x128C3)-P2-(3x256C3)-P2-2x(3x512C3-P2)-(3x4096FC), 224x224x3 -> 1000
        L = [first_layer(3, 64, 3, 1, 1), bconv(64, 64), pool(), bconv(64, 128), bconv(128, 128), pool(),
             bconv(128, 256), bconv(256, 256), bconv(256, 256), pool(),
             bconv(256, 512), bconv(512, 512), bconv(512, 512), pool(),
             bconv(512, 512), bconv(512, 512), bconv(512, 512), pool(),
             fc(7 * 7 * 512, 4096), fc(4096, 4096), fc(4096, 1000, last=True)]
        return {"layers": L, "in_hw": 224, "classes": 1000}
    raise KeyError(name)


def cnn_input(name: str, batch: int, config: int = 7) -> np.ndarray:
    hw = 32 if name.startswith("cifar") else 224
    return _rng(config, {"cifar_vgg": 1, "cifar_resnet14": 2, "alexnet": 3, "vgg16": 4}[name]).uniform(
        -1.0, 1.0, size=(batch, hw, hw, 3)).astype(np.float32)
