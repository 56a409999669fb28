"""Layer-chained forward passes of the oracle -- TEST INFRASTRUCTURE ONLY.

Compositions of the primitives in :mod:`oracle` in the order the paper's Sec. 6.1 gives for
inference (thrd -> bconv/bmm -> thrd ...), one plain call per layer, nothing fused.
Parameter containers are plain dicts of numpy arrays as produced by the seeded generators.
"""
from __future__ import annotations

import numpy as np

import oracle as orc


def mlp_forward(images_u8: np.ndarray, params: dict, keep: bool = False):
    """Binarized MLP (784-1024-1024-1024-10 in the benchmark configuration).

    images_u8 [batch][K0] uint8.  params: ``in_thr`` (int), ``W`` list of packed weights
    [N_l][ldw_l], ``K`` list of input widths, ``thr`` list of int32 thresholds for every layer but
    the last.  Layer l: v = BMM(x_{l-1}, W_l); x_l = (v >= thr_l); the last layer returns int32
    scores (Sec. 6.1: the last layer's output is not thresholded).
    Returns scores [batch][N_last] (and the list of hidden bit tensors if ``keep``).
    """
    W, K, thr = params["W"], params["K"], params["thr"]
    x = orc.pack_u8(images_u8, params["in_thr"], ldb_w=W[0].shape[1])
    hidden = []
    for l in range(len(W) - 1):
        v = orc.bmm(x, W[l], K[l])
        x = orc.threshold_pack(v, thr[l], ldb_w=W[l + 1].shape[1])
        hidden.append(x)
    scores = orc.bmm(x, W[-1], K[-1])
    return (scores, hidden) if keep else scores


def resnet18_forward(x_f32: np.ndarray, params: dict, stem_bits: np.ndarray | None = None,
                     tier: int = 0, keep: bool = False, pad_mode: int = orc.PAD_MINUS_ONE):
    """ResNet-18-shaped BNN (paper Table 5 structure 64C7/4-4x64C3-4x128C3-4x256C3-4x512C3).

    Reading used by this build (the paper leaves the details open):
      stem   : fp32 conv 7x7, stride 4, zero pad 3, 3->64; x0 = (stem >= stem_thr) (Eq. 1);
               R0 = the +1/-1 values of x0 as int32.
      block b: h = thr1(bconv3x3(x, W1, stride_b, pad 1));
               S = bconv3x3(h, W2, 1, pad 1) + shortcut,
               shortcut = R_in for stride-1 blocks, bconv1x1(x, Wd, stride 2, pad 0) for the
               three stride-2 blocks (int32); y = (S >= thr2); R_out = S.
               The residual stays full precision (Sec. 6.1), here int32, and is added before
               the threshold.  Out-of-frame inputs count as -1, or, with ``pad_mode`` =
               PAD_EXCLUDE, contribute nothing in any convolution of a block (Sec. 5.3).
      head   : pooled = sum of +1/-1 of the last y over the 7x7 positions (exact integer);
               logits = fp32 FC(pooled / 49).
    ``stem_bits`` replaces the oracle's own x0 (used to continue from the GPU's stem bits when a
    stem value sits inside the fp32 tolerance of its threshold).
    Returns logits [N][1000] fp32, or a dict of every intermediate if ``keep``.
    """
    trace = {}
    stem = orc.conv_f32(x_f32, params["stem_w"], stride=4, pad=3)
    trace["stem_f32"] = stem
    x = orc.pack_f32(stem, params["stem_thr"]) if stem_bits is None else np.ascontiguousarray(stem_bits, np.uint32)
    trace["x0"] = x
    C = params["stem_w"].shape[0]
    N, H, W_, cw = x.shape
    R = orc.unpack_pm1(x.reshape(-1, cw), C).astype(np.int32).reshape(N, H, W_, C)
    for b, blk in enumerate(params["blocks"]):
        cin, cout, stride = blk["cin"], blk["cout"], blk["stride"]
        v1 = orc.bconv(x, blk["W1"], cin, stride, 1, pad_mode, tier=tier)
        h = orc.threshold_pack(v1, blk["thr1"])
        v2 = orc.bconv(h, blk["W2"], cout, 1, 1, pad_mode, tier=tier)
        if "Wd" in blk:
            shortcut = orc.bconv(x, blk["Wd"], cin, stride, 0, pad_mode, tier=tier)     # pad 0: the modes agree
        else:
            shortcut = R
        S = v2 + shortcut
        x = orc.threshold_pack(S, blk["thr2"])
        R = S
        trace["h%d" % b] = h
        trace["y%d" % b] = x
        trace["S%d" % b] = S
    pooled = orc.sumpool_pm1(x, params["blocks"][-1]["cout"])
    trace["pooled"] = pooled
    HW = x.shape[1] * x.shape[2]
    logits = orc.head_fc_f32(pooled, params["fc_w"], float(HW))
    trace["logits"] = logits
    return trace if keep else logits


def cnn_forward(x_f32: np.ndarray, layers: list, stem_bits: np.ndarray | None = None, tier: int = 0, keep: bool = False):
    """Sequential binarized CNN in the inference order of Sec. 6.1 (thrd -> bconv -> thrd -> pool ...),
    as used for the Cifar-10 VGG / ResNet-14 and ImageNet AlexNet / VGG-16 shapes of the paper's Table 5.

    ``layers`` is a list of dicts, one per layer:
      {"op": "conv_f32", "w", "thr", "stride", "pad"}          first layer: fp32 conv (zero pad) then x >= thr
      {"op": "bwn", "W", "thr", "C", "stride", "pad"}          first layer: real input, weight bits (add / subtract)
      {"op": "bconv", "W", "thr", "C", "stride", "pad"}        binarized conv (-1 padding) + threshold
      {"op": "pool", "win", "stride"}                          max-pooling of +1/-1 values
      {"op": "block", "W1","thr1","W2","thr2",["Wd"],"cin","cout","stride"}   residual block as in resnet18_forward
      {"op": "fc", "W", "thr" | None, "K"}                      binarized FC on the flattened NHWC bits; thr None: int32 scores
    Returns the last layer's output (int32 scores), or a list with every layer's output if ``keep``.
    """
    outs = []
    x = None           # current packed activation [N][H][W][cw] or [N][ldw]
    C = 0
    R = None
    for li, L in enumerate(layers):
        op = L["op"]
        if op == "conv_f32":
            y = orc.conv_f32(x_f32, L["w"], L["stride"], L["pad"])
            x = orc.pack_f32(y, L["thr"]) if stem_bits is None else np.ascontiguousarray(stem_bits, np.uint32)
            C = L["w"].shape[0]
            R = None
            outs.append(x)
        elif op == "bwn":
            y = orc.bwn_conv_f32(x_f32, L["W"], L["C"], L["stride"], L["pad"])
            x = orc.pack_f32(y, L["thr"]) if stem_bits is None else np.ascontiguousarray(stem_bits, np.uint32)
            C = L["W"].shape[0]
            R = None
            outs.append(x)
        elif op == "bconv":
            v = orc.bconv(x, L["W"], L["C"], L["stride"], L["pad"], orc.PAD_MINUS_ONE, tier=tier)
            x = orc.threshold_pack(v, L["thr"])
            C = L["W"].shape[0]
            R = None
            outs.append(x)
        elif op == "pool":
            x = orc.maxpool_pm1(x, C, L["win"], L["stride"])
            R = None
            outs.append(x)
        elif op == "block":
            cin, cout, stride = L["cin"], L["cout"], L["stride"]
            if R is None and "Wd" not in L:
                N, H, W_, cw = x.shape
                R = orc.unpack_pm1(x.reshape(-1, cw), cin).astype(np.int32).reshape(N, H, W_, cin)
            v1 = orc.bconv(x, L["W1"], cin, stride, 1, orc.PAD_MINUS_ONE, tier=tier)
            h = orc.threshold_pack(v1, L["thr1"])
            v2 = orc.bconv(h, L["W2"], cout, 1, 1, orc.PAD_MINUS_ONE, tier=tier)
            sc = orc.bconv(x, L["Wd"], cin, stride, 0, orc.PAD_MINUS_ONE, tier=tier) if "Wd" in L else R
            S = v2 + sc
            x = orc.threshold_pack(S, L["thr2"])
            R = S
            C = cout
            outs.append(x)
        elif op == "fc":
            if x.ndim == 4:                                   # flatten NHWC: K index = (h*W + w)*C + c
                assert C % 32 == 0
                x = x.reshape(x.shape[0], -1)
            v = orc.bmm(x, L["W"], L["K"], tier=tier)
            if L["thr"] is None:
                outs.append(v)
                x = None
            else:
                x = orc.threshold_pack(v, L["thr"], ldb_w=(orc.nwords(v.shape[1]) + 3) // 4 * 4)
                C = v.shape[1]
                outs.append(x)
            R = None
        else:
            raise ValueError(op)
    return outs if keep else outs[-1]
