"""CPU oracle for the binarized FC / convolution path -- TEST INFRASTRUCTURE ONLY.

Thin numpy front end over ``bnn_oracle.c`` (plain C, naive loops on unpacked +1/-1 values) plus
the layer compositions in :mod:`oracle.nets`.  Nothing under ``paper_2006_16578_amd`` imports this
package, and this package imports nothing from it; only ``tests/``, ``__graft_entry__.smoke()``
and ``bench.py``'s ``cpu_baseline`` leg may use it.

Conventions (paper Sec. 5.2, Eq. 1-2): bit 1 is +1, bit 0 is -1; element k sits in word k // 32,
bit k % 32 from the least significant bit; pad bits are 0.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bnn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

PAD_MINUS_ONE = 0   # out-of-frame input counts as -1
PAD_EXCLUDE = 1     # out-of-frame taps contribute nothing (paper Sec. 5.3)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2 -fopenmp, no target-specific flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(v) -> ctypes.c_int64:
    return ctypes.c_int64(int(v))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError("oracle %s failed with status %d" % (what, rc))


def _words(a, ndim: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.uint32)
    assert a.ndim == ndim, (a.shape, ndim)
    return a


def nwords(nbits: int) -> int:
    return (int(nbits) + 31) // 32


# ----------------------------------------------------------------------------- O1
def unpack_pm1(bits, cols: int) -> np.ndarray:
    """bits [rows][ldw] uint32 -> int8 [rows][cols] in {+1, -1}."""
    bits = _words(bits, 2)
    rows, ldw = bits.shape
    out = np.empty((rows, cols), dtype=np.int8)
    _check(lib().orc_unpack_pm1(_p(bits), _i64(rows), _i64(cols), _i64(ldw), _p(out)), "unpack")
    return out


# ----------------------------------------------------------------------------- O2
def bmm(A, B, K: int, tier: int = 0) -> np.ndarray:
    """C[i][j] = sum_k a[i][k] b[j][k] over +1/-1; A [M][lda_w], B [N][ldb_w] packed along K."""
    A = _words(A, 2)
    B = _words(B, 2)
    M, lda = A.shape
    N, ldb = B.shape
    C = np.empty((M, N), dtype=np.int32)
    fn = lib().orc_bmm if tier == 0 else lib().orc1_bmm
    _check(fn(_p(A), _p(B), _p(C), _i64(M), _i64(N), _i64(K), _i64(lda), _i64(ldb), _i64(N)), "bmm")
    return C


def bmm_rows(A, B, K: int, row0: int, rows: int) -> np.ndarray:
    """Tier-0 product for rows [row0, row0+rows) of A only."""
    A = _words(A, 2)
    B = _words(B, 2)
    N = B.shape[0]
    assert 0 <= row0 and row0 + rows <= A.shape[0]
    C = np.empty((rows, N), dtype=np.int32)
    _check(lib().orc_bmm_rows(_p(A), _p(B), _p(C), _i64(row0), _i64(rows), _i64(N), _i64(K),
                              _i64(A.shape[1]), _i64(B.shape[1])), "bmm_rows")
    return C


def tile_b(B) -> np.ndarray:
    """The pre-tiled weight layout as its definition: rows grouped by 32, 16-byte unit u of row r moves to unit
    ((r // 32) * units_per_row + u) * 32 + r % 32; rows past N are zeros.  A pure permutation, no arithmetic."""
    B = _words(B, 2)
    N, ldw = B.shape
    assert ldw % 4 == 0
    upr = ldw // 4
    groups = (N + 31) // 32
    padded = np.zeros((groups * 32, upr, 4), dtype=np.uint32)
    padded[:N] = B.reshape(N, upr, 4)
    # [group][row-in-group][unit][4] -> [group][unit][row-in-group][4]
    return np.ascontiguousarray(padded.reshape(groups, 32, upr, 4).transpose(0, 2, 1, 3)).reshape(groups * 32, ldw)


def panels(X, K: int) -> np.ndarray:
    """The K-panel layout as its definition: K cut into panels of 256 bits, panel p holding words 8p .. 8p+7 of every
    row back to back, [ceil(K/256)][rows][8]; bits past K are 0.  A pure permutation, no arithmetic."""
    X = _words(X, 2)
    rows, ldw = X.shape
    kw = (K + 31) // 32
    assert ldw >= kw
    npan = (K + 255) // 256
    padded = np.zeros((rows, npan * 8), dtype=np.uint32)
    padded[:, :kw] = X[:, :kw]
    if K % 32:
        padded[:, kw - 1] &= np.uint32((1 << (K % 32)) - 1)
    return np.ascontiguousarray(padded.reshape(rows, npan, 8).transpose(1, 0, 2))


# ----------------------------------------------------------------------------- O3
def conv_out_size(H: int, k: int, stride: int, pad: int) -> int:
    return (H + 2 * pad - k) // stride + 1


def bconv(x, filt, C: int, stride: int, pad: int, pad_mode: int = PAD_MINUS_ONE, tier: int = 0) -> np.ndarray:
    """x [N][H][W][cw], filt [O][k][k][cw] packed along C -> int32 [N][P][Q][O]."""
    x = _words(x, 4)
    filt = _words(filt, 4)
    N, H, W, cw = x.shape
    O, k, k2, cwf = filt.shape
    assert k == k2 and cw == cwf == nwords(C), (x.shape, filt.shape, C)
    P, Q = conv_out_size(H, k, stride, pad), conv_out_size(W, k, stride, pad)
    out = np.empty((N, P, Q, O), dtype=np.int32)
    fn = lib().orc_bconv if tier == 0 else lib().orc1_bconv
    _check(fn(_p(x), _p(filt), _p(out), _i64(N), _i64(H), _i64(W), _i64(C), _i64(O), _i64(k),
              _i64(stride), _i64(pad), ctypes.c_int(pad_mode)), "bconv")
    return out


def bconv_images(x, filt, C: int, stride: int, pad: int, pad_mode: int, n0: int, n_cnt: int) -> np.ndarray:
    """Tier-0 convolution of images [n0, n0+n_cnt) only."""
    x = _words(x, 4)
    filt = _words(filt, 4)
    N, H, W, cw = x.shape
    O, k, _, _ = filt.shape
    assert 0 <= n0 and n0 + n_cnt <= N
    P, Q = conv_out_size(H, k, stride, pad), conv_out_size(W, k, stride, pad)
    out = np.empty((n_cnt, P, Q, O), dtype=np.int32)
    _check(lib().orc_bconv_images(_p(x), _p(filt), _p(out), _i64(n0), _i64(n_cnt), _i64(H), _i64(W),
                                  _i64(C), _i64(O), _i64(k), _i64(stride), _i64(pad),
                                  ctypes.c_int(pad_mode)), "bconv_images")
    return out


# ----------------------------------------------------------------------------- O4
def threshold_pack(X, tau, ldb_w: int | None = None) -> np.ndarray:
    """int32 [..., cols] with tau [cols] -> bits [..., ldb_w]; bit = (v >= tau)."""
    X = np.ascontiguousarray(X, dtype=np.int32)
    tau = np.ascontiguousarray(tau, dtype=np.int32)
    cols = X.shape[-1]
    assert tau.shape == (cols,)
    rows = int(np.prod(X.shape[:-1], dtype=np.int64))
    ldb_w = nwords(cols) if ldb_w is None else ldb_w
    bits = np.empty((rows, ldb_w), dtype=np.uint32)
    _check(lib().orc_threshold_pack(_p(X), _p(tau), _p(bits), _i64(rows), _i64(cols), _i64(cols),
                                    _i64(ldb_w)), "threshold_pack")
    return bits.reshape(X.shape[:-1] + (ldb_w,))


def pack_u8(x, thr: int, ldb_w: int | None = None) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint8)
    assert x.ndim == 2
    rows, cols = x.shape
    ldb_w = nwords(cols) if ldb_w is None else ldb_w
    bits = np.empty((rows, ldb_w), dtype=np.uint32)
    _check(lib().orc_pack_u8(_p(x), ctypes.c_int(thr), _p(bits), _i64(rows), _i64(cols), _i64(ldb_w)), "pack_u8")
    return bits


def pack_f32(x, tau, ldb_w: int | None = None) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    cols = x.shape[-1]
    assert tau.shape == (cols,)
    rows = int(np.prod(x.shape[:-1], dtype=np.int64))
    ldb_w = nwords(cols) if ldb_w is None else ldb_w
    bits = np.empty((rows, ldb_w), dtype=np.uint32)
    _check(lib().orc_pack_f32(_p(x), _p(tau), _p(bits), _i64(rows), _i64(cols), _i64(ldb_w)), "pack_f32")
    return bits.reshape(x.shape[:-1] + (ldb_w,))


def maxpool_pm1(bits, C: int, win: int, stride: int) -> np.ndarray:
    """bits [N][H][W][cw] -> [N][P][Q][cw]: maximum of the +1/-1 values over win x win windows."""
    bits = _words(bits, 4)
    N, H, W, cw = bits.shape
    assert cw == nwords(C)
    P, Q = (H - win) // stride + 1, (W - win) // stride + 1
    out = np.empty((N, P, Q, cw), dtype=np.uint32)
    _check(lib().orc_maxpool_pm1(_p(bits), _p(out), _i64(N), _i64(H), _i64(W), _i64(C), _i64(win), _i64(stride)),
           "maxpool")
    return out


# ----------------------------------------------------------------------------- fp32 ends
def conv_f32(x, w, stride: int, pad: int) -> np.ndarray:
    """x [N][H][W][C] fp32 (zero padded), w [O][k][k][C] -> fp32 [N][P][Q][O]; double accumulation."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, H, W, C = x.shape
    O, k, k2, C2 = w.shape
    assert k == k2 and C == C2
    P, Q = conv_out_size(H, k, stride, pad), conv_out_size(W, k, stride, pad)
    y = np.empty((N, P, Q, O), dtype=np.float32)
    _check(lib().orc_conv_f32(_p(x), _p(w), _p(y), _i64(N), _i64(H), _i64(W), _i64(C), _i64(O),
                              _i64(k), _i64(stride), _i64(pad)), "conv_f32")
    return y


def bwn_conv_f32(x, wbits, C: int, stride: int, pad: int) -> np.ndarray:
    """First layer with binarized weights (Sec. 6.1): x [N][H][W][C] fp32 (zero padded), wbits [O][k][k][cw]
    -> fp32 [N][P][Q][O]; each input element is added or subtracted according to its weight bit."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    wbits = _words(wbits, 4)
    N, H, W, C2 = x.shape
    O, k, k2, cw = wbits.shape
    assert k == k2 and C == C2 and cw == nwords(C)
    P, Q = conv_out_size(H, k, stride, pad), conv_out_size(W, k, stride, pad)
    y = np.empty((N, P, Q, O), dtype=np.float32)
    _check(lib().orc_bwn_conv_f32(_p(x), _p(wbits), _p(y), _i64(N), _i64(H), _i64(W), _i64(C), _i64(O),
                                  _i64(k), _i64(stride), _i64(pad)), "bwn_conv_f32")
    return y


def general_bmm_f32(A, B) -> np.ndarray:
    """The "general" BMM of Sec. 7.2: real-valued A [M][K] and B [N][K] are binarized by Eq. 1 (x >= 0 -> +1),
    multiplied as +1/-1 matrices (Eq. 2), and the result is returned as real values [M][N]."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    K = A.shape[1]
    assert B.shape[1] == K
    zero = np.zeros(K, dtype=np.float32)
    return bmm(pack_f32(A, zero), pack_f32(B, zero), K).astype(np.float32)


def general_bconv_f32(x, filt, stride: int, pad: int, pad_mode: int = PAD_MINUS_ONE) -> np.ndarray:
    """The "general" BConv of Sec. 7.3: real-valued x [N][H][W][C] and filt [O][k][k][C] are binarized by
    Eq. 1, convolved as +1/-1 tensors, and the result is returned as real values [N][P][Q][O]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    filt = np.ascontiguousarray(filt, dtype=np.float32)
    C = x.shape[-1]
    zero = np.zeros(C, dtype=np.float32)
    return bconv(pack_f32(x, zero), pack_f32(filt, zero), C, stride, pad, pad_mode).astype(np.float32)


def sumpool_pm1(bits, C: int) -> np.ndarray:
    """bits [N][H][W][cw] -> int32 [N][C]: sum of +1/-1 over all H*W positions."""
    bits = _words(bits, 4)
    N, H, W, cw = bits.shape
    assert cw == nwords(C)
    pooled = np.empty((N, C), dtype=np.int32)
    _check(lib().orc_sumpool_pm1(_p(bits), _p(pooled), _i64(N), _i64(H * W), _i64(C)), "sumpool")
    return pooled


def head_fc_f32(pooled, w, div: float) -> np.ndarray:
    pooled = np.ascontiguousarray(pooled, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, C = pooled.shape
    J, C2 = w.shape
    assert C == C2
    y = np.empty((N, J), dtype=np.float32)
    _check(lib().orc_head_fc_f32(_p(pooled), _p(w), _p(y), _i64(N), _i64(C), _i64(J),
                                 ctypes.c_float(div)), "head_fc")
    return y
