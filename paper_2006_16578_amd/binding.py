"""ctypes binding of libbnn's C ABI (include/bnn.h): argument marshalling only.

Tensors are ``torch`` CUDA (ROCm) tensors used purely as device buffers; every function enqueues
on torch's current stream of the tensor's device and returns the output tensor(s).  Shapes and
dtypes are checked here, everything else by the library, whose status codes are raised as
``BnnError``.
"""
from __future__ import annotations

import ctypes
import os

import torch

__all__ = ["BnnError", "lib_path", "load", "PAD_MINUS_ONE", "PAD_EXCLUDE", "PATH_AUTO", "PATH_VALU", "PATH_MFMA",
           "nwords", "round_up", "bmm", "bmm_thr", "bconv", "bconv_thr", "threshold_pack", "pack_u8", "pack_f32",
           "unpack_i32", "tile_b", "bmm_tiled", "bmm_thr_tiled", "panels_from_rows", "rows_from_panels", "bmm_panels", "bmm_thr_panels", "probe_load_stride", "probe_pipeline", "probe_pipeline_enqueue", "PROBES", "sign_pack_f32", "bmm_general_f32", "bconv_general_f32", "maxpool_or", "conv_f32_thr", "conv_f32_split_thr", "bwn_conv_thr", "head_f32", "Net", "EXPORTS", "bmm_kernel_name", "bconv_kernel_name"]

PAD_MINUS_ONE, PAD_EXCLUDE = 0, 1
PATH_AUTO, PATH_VALU, PATH_MFMA = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))

# every symbol include/bnn.h declares
EXPORTS = ["bnn_status_string", "bnn_version", "bnn_bmm_kernel_name", "bnn_bconv_kernel_name", "bnn_bmm_kernel_name_out", "bnn_bconv_kernel_name_out", "bnn_bmm", "bnn_bmm_ex", "bnn_bmm_thr", "bnn_bmm_thr_ex",
           "bnn_bconv", "bnn_bconv_ex", "bnn_bconv_thr", "bnn_bconv_thr_ex", "bnn_threshold_pack", "bnn_pack_u8",
           "bnn_pack_f32", "bnn_tile_b", "bnn_bmm_tiled", "bnn_bmm_thr_tiled", "bnn_panels_from_rows", "bnn_rows_from_panels", "bnn_bmm_panels", "bnn_bmm_thr_panels", "bnn_probe_load_stride", "bnn_probe_pipeline", "bnn_sign_pack_f32", "bnn_bmm_general_workspace_bytes", "bnn_bmm_general_f32",
           "bnn_bconv_general_workspace_bytes", "bnn_bconv_general_f32", "bnn_unpack_i32", "bnn_maxpool_or", "bnn_conv_f32_thr", "bnn_conv_f32_split_workspace_bytes", "bnn_conv_f32_split_thr", "bnn_conv_f32_split_thr_ex", "bnn_bwn_workspace_bytes", "bnn_bwn_conv_thr", "bnn_head_f32", "bnn_net_create",
           "bnn_net_destroy", "bnn_net_input_u8", "bnn_net_input_bits", "bnn_net_input_conv_f32", "bnn_net_input_bwn_f32", "bnn_net_add_fc",
           "bnn_net_add_conv", "bnn_net_add_pool", "bnn_net_add_block", "bnn_net_add_head_f32", "bnn_net_workspace_bytes",
           "bnn_net_forward", "bnn_net_forward_static", "bnn_static_workspace_init", "bnn_net_forward_persistent", "bnn_net_persistent_status", "bnn_net_layer_bits"]


class BnnError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, _status_string(status), status))


def lib_path() -> str:
    return os.path.join(_HERE, "libbnn.so")


_lib = None


def load() -> ctypes.CDLL:
    """Loads libbnn.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError("libbnn.so is not built: run `python -m paper_2006_16578_amd.build` "
                              "(or __graft_entry__.build()) first")
        lib = ctypes.CDLL(path)
        lib.bnn_status_string.restype = ctypes.c_char_p
        lib.bnn_status_string.argtypes = [ctypes.c_int]
        lib.bnn_bmm_kernel_name.restype = ctypes.c_char_p
        lib.bnn_bconv_kernel_name.restype = ctypes.c_char_p
        lib.bnn_bmm_kernel_name_out.restype = ctypes.c_char_p
        lib.bnn_bconv_kernel_name_out.restype = ctypes.c_char_p
        lib.bnn_bwn_workspace_bytes.restype = ctypes.c_size_t
        lib.bnn_conv_f32_split_workspace_bytes.restype = ctypes.c_size_t
        lib.bnn_bmm_general_workspace_bytes.restype = ctypes.c_size_t
        lib.bnn_bconv_general_workspace_bytes.restype = ctypes.c_size_t
        for name in EXPORTS:
            getattr(lib, name)          # fail loudly on a missing export
        _lib = lib
    return _lib


def _status_string(status: int) -> str:
    try:
        return load().bnn_status_string(status).decode()
    except Exception:  # pragma: no cover
        return "?"


def _check(status: int, what: str) -> None:
    if status != 0:
        raise BnnError(status, what)


def bmm_kernel_name(M: int, N: int, K: int, path: int = PATH_AUTO, int32_out: bool = False) -> str:
    return load().bnn_bmm_kernel_name_out(int(M), int(N), int(K), int(path), int(bool(int32_out))).decode()


def bconv_kernel_name(N, H, W, C, O, k, stride, pad, path: int = PATH_AUTO, int32_out: bool = False) -> str:
    return load().bnn_bconv_kernel_name_out(int(N), int(H), int(W), int(C), int(O), int(k), int(stride), int(pad),
                                            int(path), int(bool(int32_out))).decode()


def nwords(nbits: int) -> int:
    return (int(nbits) + 31) // 32


def round_up(v: int, m: int) -> int:
    return (int(v) + m - 1) // m * m


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _dev(t: torch.Tensor, dtype, ndim=None, name="tensor"):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if ndim is not None and t.dim() != ndim:
        raise ValueError("%s must have %d dimensions" % (name, ndim))
    return t


_BITS = torch.int32   # packed words travel as int32 tensors (torch has no uint32 arithmetic; only the bytes matter)


def bmm(A, B, K: int, out=None, path: int = PATH_AUTO):
    """C[i][j] = sum_k a[i][k] b[j][k]; A [M][lda_w], B [N][ldb_w] packed int32 words -> int32 [M][N]."""
    _dev(A, _BITS, 2, "A"); _dev(B, _BITS, 2, "B")
    M, lda = A.shape
    N, ldb = B.shape
    C = torch.empty((M, N), dtype=torch.int32, device=A.device) if out is None else _dev(out, torch.int32, 2, "out")
    with torch.cuda.device(A.device):
        _check(load().bnn_bmm_ex(_ptr(A), _ptr(B), _ptr(C), M, N, int(K), lda, ldb, C.shape[1], int(path), _stream(A)), "bnn_bmm")
    return C


def bmm_thr(A, B, thr, K: int, ldcb_w: int | None = None, out=None, path: int = PATH_AUTO):
    """Fused BMM + threshold: bits [M][ldcb_w], bit j = (C[i][j] >= thr[j])."""
    _dev(A, _BITS, 2, "A"); _dev(B, _BITS, 2, "B"); _dev(thr, torch.int32, 1, "thr")
    M, lda = A.shape
    N, ldb = B.shape
    if thr.shape[0] != N:
        raise ValueError("thr must have N entries")
    ldcb_w = round_up(nwords(N), 4) if ldcb_w is None else int(ldcb_w)
    Cb = torch.empty((M, ldcb_w), dtype=_BITS, device=A.device) if out is None else _dev(out, _BITS, 2, "out")
    with torch.cuda.device(A.device):
        _check(load().bnn_bmm_thr_ex(_ptr(A), _ptr(B), _ptr(thr), _ptr(Cb), M, N, int(K), lda, ldb, Cb.shape[1], int(path),
                                     _stream(A)), "bnn_bmm_thr")
    return Cb


def _conv_dims(x, filt, C, stride, pad):
    _dev(x, _BITS, 4, "x"); _dev(filt, _BITS, 4, "filt")
    N, H, W, cw = x.shape
    O, k, k2, cwf = filt.shape
    if k != k2 or cw != cwf or cw != nwords(C):
        raise ValueError("x [N][H][W][cw], filt [O][k][k][cw] with cw = ceil(C/32) expected")
    if stride < 1:                       # the library rejects it; keep the shapes computable
        return N, H, W, O, k, 1, 1
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    return N, H, W, O, k, P, Q


def bconv(x, filt, C: int, stride: int, pad: int, pad_mode: int = PAD_MINUS_ONE, out=None, path: int = PATH_AUTO):
    """int32 [N][P][Q][O] = cross-correlation of packed x [N][H][W][cw] with filt [O][k][k][cw]."""
    N, H, W, O, k, P, Q = _conv_dims(x, filt, C, stride, pad)
    y = torch.empty((N, max(P, 0), max(Q, 0), O), dtype=torch.int32, device=x.device) if out is None else out
    with torch.cuda.device(x.device):
        _check(load().bnn_bconv_ex(_ptr(x), _ptr(filt), _ptr(y), N, H, W, int(C), O, k, int(stride), int(pad),
                                   int(pad_mode), int(path), _stream(x)), "bnn_bconv")
    return y


def bconv_thr(x, filt, thr, C: int, stride: int, pad: int, pad_mode: int = PAD_MINUS_ONE, residual=None,
              want_sum: bool = False, sum_out=None, out=None, path: int = PATH_AUTO):
    """Fused conv (+ int32 residual) + threshold -> bits [N][P][Q][ow]; optionally also the int32 sum."""
    N, H, W, O, k, P, Q = _conv_dims(x, filt, C, stride, pad)
    _dev(thr, torch.int32, 1, "thr")
    if residual is not None:
        _dev(residual, torch.int32, 4, "residual")
        if tuple(residual.shape) != (N, P, Q, O):
            raise ValueError("residual must be [N][P][Q][O]")
    if want_sum and sum_out is None:
        sum_out = torch.empty((N, P, Q, O), dtype=torch.int32, device=x.device)
    bits = torch.empty((N, max(P, 0), max(Q, 0), nwords(O)), dtype=_BITS, device=x.device) if out is None else out
    with torch.cuda.device(x.device):
        _check(load().bnn_bconv_thr_ex(_ptr(x), _ptr(filt), _ptr(residual), _ptr(sum_out), _ptr(thr), _ptr(bits), N, H, W,
                                       int(C), O, k, int(stride), int(pad), int(pad_mode), int(path), _stream(x)),
               "bnn_bconv_thr")
    return (bits, sum_out) if sum_out is not None else bits


def threshold_pack(X, thr, ldb_w: int | None = None):
    _dev(X, torch.int32, None, "X"); _dev(thr, torch.int32, 1, "thr")
    cols = X.shape[-1]
    rows = X.numel() // cols
    ldb_w = nwords(cols) if ldb_w is None else int(ldb_w)
    bits = torch.empty(tuple(X.shape[:-1]) + (ldb_w,), dtype=_BITS, device=X.device)
    with torch.cuda.device(X.device):
        _check(load().bnn_threshold_pack(_ptr(X), _ptr(thr), _ptr(bits), ctypes.c_int64(rows), cols, cols, ldb_w, _stream(X)),
               "bnn_threshold_pack")
    return bits


def pack_u8(x, thr: int, ldb_w: int | None = None):
    _dev(x, torch.uint8, 2, "x")
    rows, cols = x.shape
    ldb_w = nwords(cols) if ldb_w is None else int(ldb_w)
    bits = torch.empty((rows, ldb_w), dtype=_BITS, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().bnn_pack_u8(_ptr(x), int(thr), _ptr(bits), ctypes.c_int64(rows), cols, ldb_w, _stream(x)), "bnn_pack_u8")
    return bits


def pack_f32(x, thr, ldb_w: int | None = None):
    _dev(x, torch.float32, None, "x"); _dev(thr, torch.float32, 1, "thr")
    cols = x.shape[-1]
    rows = x.numel() // cols
    ldb_w = nwords(cols) if ldb_w is None else int(ldb_w)
    bits = torch.empty(tuple(x.shape[:-1]) + (ldb_w,), dtype=_BITS, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().bnn_pack_f32(_ptr(x), _ptr(thr), _ptr(bits), ctypes.c_int64(rows), cols, ldb_w, _stream(x)), "bnn_pack_f32")
    return bits


def tile_b(B, K: int):
    """Weights [N][ldb_w] -> the pre-tiled layout bnn_bmm_tiled reads (32-row groups, 16-byte units interleaved)."""
    _dev(B, _BITS, 2, "B")
    N, ldb = B.shape
    out = torch.empty(((N + 31) // 32 * 32, ldb), dtype=_BITS, device=B.device)
    with torch.cuda.device(B.device):
        _check(load().bnn_tile_b(_ptr(B), _ptr(out), N, int(K), ldb, _stream(B)), "bnn_tile_b")
    return out


def bmm_tiled(A, Bt, N: int, K: int, out=None):
    _dev(A, _BITS, 2, "A"); _dev(Bt, _BITS, 2, "Bt")
    M = A.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    with torch.cuda.device(A.device):
        _check(load().bnn_bmm_tiled(_ptr(A), _ptr(Bt), _ptr(out), M, int(N), int(K), A.shape[1], Bt.shape[1], out.shape[1],
                                    _stream(A)), "bnn_bmm_tiled")
    return out


def bmm_thr_tiled(A, Bt, thr, N: int, K: int, ldcb_w: int | None = None, out=None):
    _dev(A, _BITS, 2, "A"); _dev(Bt, _BITS, 2, "Bt"); _dev(thr, torch.int32, 1, "thr")
    M = A.shape[0]
    ldcb_w = round_up(nwords(N), 4) if ldcb_w is None else ldcb_w
    if out is None:
        out = torch.empty((M, ldcb_w), dtype=_BITS, device=A.device)
    with torch.cuda.device(A.device):
        _check(load().bnn_bmm_thr_tiled(_ptr(A), _ptr(Bt), _ptr(thr), _ptr(out), M, int(N), int(K), A.shape[1], Bt.shape[1],
                                        out.shape[1], _stream(A)), "bnn_bmm_thr_tiled")
    return out


def panels_from_rows(X, K: int):
    """Packed [rows][ldx_w] -> the K-panel layout ([ceil(K/256)][rows][8] words) that bmm_panels / bmm_thr_panels read."""
    _dev(X, _BITS, 2, "X")
    rows, ldx = X.shape
    out = torch.empty(((int(K) + 255) // 256, rows, 8), dtype=_BITS, device=X.device)
    with torch.cuda.device(X.device):
        _check(load().bnn_panels_from_rows(_ptr(X), _ptr(out), ctypes.c_int64(rows), int(K), ldx, _stream(X)), "bnn_panels_from_rows")
    return out


def rows_from_panels(Xp, K: int, ldx_w: int | None = None):
    """The K-panel layout back to packed rows [rows][ldx_w]."""
    _dev(Xp, _BITS, 3, "Xp")
    rows = Xp.shape[1]
    ldx_w = round_up(nwords(K), 4) if ldx_w is None else int(ldx_w)
    out = torch.empty((rows, ldx_w), dtype=_BITS, device=Xp.device)
    with torch.cuda.device(Xp.device):
        _check(load().bnn_rows_from_panels(_ptr(Xp), _ptr(out), ctypes.c_int64(rows), int(K), ldx_w, _stream(Xp)), "bnn_rows_from_panels")
    return out


def bmm_panels(Ap, Bp, K: int, out=None):
    """int32 [M][N] = A x B^T with both operands in K panels ([panels][rows][8])."""
    _dev(Ap, _BITS, 3, "Ap"); _dev(Bp, _BITS, 3, "Bp")
    M, N = Ap.shape[1], Bp.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=Ap.device)
    with torch.cuda.device(Ap.device):
        _check(load().bnn_bmm_panels(_ptr(Ap), _ptr(Bp), _ptr(out), M, N, int(K), out.shape[1], _stream(Ap)), "bnn_bmm_panels")
    return out


def bmm_thr_panels(Ap, Bp, thr, K: int, out=None):
    """Fused threshold; the output bits come in K panels ([ceil(N/256)][M][8]), the next product's A."""
    _dev(Ap, _BITS, 3, "Ap"); _dev(Bp, _BITS, 3, "Bp"); _dev(thr, torch.int32, 1, "thr")
    M, N = Ap.shape[1], Bp.shape[1]
    if out is None:
        out = torch.empty(((N + 255) // 256, M, 8), dtype=_BITS, device=Ap.device)
    with torch.cuda.device(Ap.device):
        _check(load().bnn_bmm_thr_panels(_ptr(Ap), _ptr(Bp), _ptr(thr), _ptr(out), M, N, int(K), _stream(Ap)), "bnn_bmm_thr_panels")
    return out


def probe_load_stride(stride_bytes: int, rows: int | None = None, iters: int = 4096, dependent: bool = True, device="cuda",
                      footprint_bytes: int = 1 << 20):
    """Shader-cycle-counter ticks per MFMA operand-fragment load of one wave, rows `stride_bytes` apart (diagnostic).
    By default the buffer is `footprint_bytes` in all, so that every stride is measured at the same cache level."""
    if rows is None:
        rows = max(32, footprint_bytes // stride_bytes // 32 * 32)
    buf = torch.zeros(rows * stride_bytes // 4, dtype=_BITS, device=device)
    cyc = torch.zeros(2, dtype=torch.int64, device=device)
    with torch.cuda.device(buf.device):
        for _ in range(2):                                  # the second run has the buffer in cache
            _check(load().bnn_probe_load_stride(_ptr(buf), _ptr(cyc), int(stride_bytes), int(rows), int(iters),
                                                1 if dependent else 0, _stream(buf)), "bnn_probe_load_stride")
    return float(cyc[0].item()) / iters


PROBES = {"mfma_fp4": 0, "mfma_fp4_expand": 1, "mfma_i8": 2, "mfma_bf16": 3, "valu_xor_popc": 4, "lds_read": 5,
          "hbm_read": 6, "hbm_write": 7, "hbm_copy": 8}


def probe_pipeline(which: str, buf, iters: int = 2000, reps: int = 3):
    """Runs one ceiling microbenchmark (bnn_probe_pipeline) `reps` times after a warm-up launch; returns
    (work units per second of the fastest launch, seconds of that launch).  buf: a uint8 device tensor."""
    _dev(buf, torch.uint8, 1, "buf")
    work = ctypes.c_double(0.0)
    best = None
    with torch.cuda.device(buf.device):
        for rep in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            _check(load().bnn_probe_pipeline(PROBES[which], _ptr(buf), ctypes.c_size_t(buf.numel()), int(iters),
                                             ctypes.byref(work), _stream(buf)), "bnn_probe_pipeline")
            e1.record()
            e1.synchronize()
            sec = e0.elapsed_time(e1) * 1e-3
            if rep > 0 and (best is None or sec < best):
                best = sec
    return work.value / best, best


def probe_pipeline_enqueue(which: str, buf, iters: int) -> float:
    """Enqueues one launch of a ceiling microbenchmark without waiting for it; returns its work units."""
    _dev(buf, torch.uint8, 1, "buf")
    work = ctypes.c_double(0.0)
    with torch.cuda.device(buf.device):
        _check(load().bnn_probe_pipeline(PROBES[which], _ptr(buf), ctypes.c_size_t(buf.numel()), int(iters),
                                         ctypes.byref(work), _stream(buf)), "bnn_probe_pipeline")
    return work.value


def sign_pack_f32(x, ldb_w: int | None = None):
    """Binarization by sign: x [rows][cols] fp32 -> bits [rows][ldb_w], bit = (x >= 0)."""
    _dev(x, torch.float32, 2, "x")
    rows, cols = x.shape
    ldb_w = nwords(cols) if ldb_w is None else ldb_w
    bits = torch.empty((rows, ldb_w), dtype=_BITS, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().bnn_sign_pack_f32(_ptr(x), _ptr(bits), ctypes.c_int64(rows), cols, cols, ldb_w, _stream(x)), "bnn_sign_pack_f32")
    return bits


def bmm_general_f32(A, B, out=None, workspace=None):
    """General BMM: fp32 A [M][K], B [N][K] -> fp32 [M][N] of the sign-binarized product."""
    _dev(A, torch.float32, 2, "A"); _dev(B, torch.float32, 2, "B")
    M, K = A.shape
    N = B.shape[0]
    if B.shape[1] != K:
        raise ValueError("K mismatch")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    if workspace is None:
        workspace = torch.empty(max(int(load().bnn_bmm_general_workspace_bytes(M, N, K)), 256), dtype=torch.uint8, device=A.device)
    with torch.cuda.device(A.device):
        _check(load().bnn_bmm_general_f32(_ptr(A), _ptr(B), _ptr(out), M, N, K, K, K, N, _ptr(workspace),
                                          ctypes.c_size_t(workspace.numel()), _stream(A)), "bnn_bmm_general_f32")
    return out


def bconv_general_f32(x, filt, stride: int, pad: int, pad_mode: int = PAD_MINUS_ONE, out=None, workspace=None):
    """General BConv: fp32 x [N][H][W][C], filt [O][k][k][C] -> fp32 [N][P][Q][O] of the sign-binarized convolution."""
    _dev(x, torch.float32, 4, "x"); _dev(filt, torch.float32, 4, "filt")
    N, H, W, C = x.shape
    O, k, _, C2 = filt.shape
    if C != C2:
        raise ValueError("channel mismatch")
    P = (H + 2 * pad - k) // stride + 1 if stride > 0 else 1
    Q = (W + 2 * pad - k) // stride + 1 if stride > 0 else 1
    if out is None:
        out = torch.empty((N, max(P, 1), max(Q, 1), O), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(int(load().bnn_bconv_general_workspace_bytes(N, H, W, C, O, k)), 256), dtype=torch.uint8,
                                device=x.device)
    with torch.cuda.device(x.device):
        _check(load().bnn_bconv_general_f32(_ptr(x), _ptr(filt), _ptr(out), N, H, W, C, O, k, int(stride), int(pad), int(pad_mode),
                                            _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(x)), "bnn_bconv_general_f32")
    return out


def unpack_i32(bits, cols: int):
    _dev(bits, _BITS, None, "bits")
    ldb_w = bits.shape[-1]
    rows = bits.numel() // ldb_w
    out = torch.empty(tuple(bits.shape[:-1]) + (cols,), dtype=torch.int32, device=bits.device)
    with torch.cuda.device(bits.device):
        _check(load().bnn_unpack_i32(_ptr(bits), _ptr(out), ctypes.c_int64(rows), int(cols), ldb_w, int(cols), _stream(bits)),
               "bnn_unpack_i32")
    return out


def maxpool_or(bits, C: int, win: int, stride: int):
    """bits [N][H][W][cw] -> [N][P][Q][cw]: max-pooling of +1/-1 activations as a bitwise OR."""
    _dev(bits, _BITS, 4, "bits")
    N, H, W, cw = bits.shape
    ok = stride >= 1 and 1 <= win <= min(H, W)          # anything else is left for the library to reject
    P, Q = ((H - win) // stride + 1, (W - win) // stride + 1) if ok else (1, 1)
    out = torch.empty((N, P, Q, cw), dtype=_BITS, device=bits.device)
    with torch.cuda.device(bits.device):
        _check(load().bnn_maxpool_or(_ptr(bits), _ptr(out), N, H, W, int(C), int(win), int(stride), _stream(bits)),
               "bnn_maxpool_or")
    return out


def conv_f32_thr(x, w, thr, stride: int, pad: int, want_f32: bool = False):
    """fp32 first layer: x [N][H][W][C], w [O][k][k][C], thr [O] -> bits [N][P][Q][ow] (and fp32 y)."""
    _dev(x, torch.float32, 4, "x"); _dev(w, torch.float32, 4, "w"); _dev(thr, torch.float32, 1, "thr")
    N, H, W, C = x.shape
    O, k, _, C2 = w.shape
    if C != C2:
        raise ValueError("channel mismatch")
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    bits = torch.empty((N, P, Q, nwords(O)), dtype=_BITS, device=x.device)
    y = torch.empty((N, P, Q, O), dtype=torch.float32, device=x.device) if want_f32 else None
    with torch.cuda.device(x.device):
        _check(load().bnn_conv_f32_thr(_ptr(x), _ptr(w), _ptr(thr), _ptr(y), _ptr(bits), N, H, W, C, O, k, int(stride), int(pad),
                                       _stream(x)), "bnn_conv_f32_thr")
    return (bits, y) if want_f32 else bits


def conv_f32_split_thr(x, w, thr, stride: int, pad: int, want_f32: bool = False, workspace=None, products: int = 9):
    """fp32 first layer on the bf16 matrix cores (inputs and weights split exactly into three bf16 terms each;
    products: 9 term products, or 6 without the three smallest)."""
    _dev(x, torch.float32, 4, "x"); _dev(w, torch.float32, 4, "w"); _dev(thr, torch.float32, 1, "thr")
    N, H, W, C = x.shape
    O, k, _, C2 = w.shape
    if C != C2:
        raise ValueError("channel mismatch")
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    bits = torch.empty((N, P, Q, nwords(O)), dtype=_BITS, device=x.device)
    y = torch.empty((N, P, Q, O), dtype=torch.float32, device=x.device) if want_f32 else None
    if workspace is None:
        workspace = torch.empty(max(int(load().bnn_conv_f32_split_workspace_bytes(C, O, k)), 16), dtype=torch.uint8, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().bnn_conv_f32_split_thr_ex(_ptr(x), _ptr(w), _ptr(thr), _ptr(y), _ptr(bits), N, H, W, C, O, k, int(stride),
                                                int(pad), int(products), _ptr(workspace), ctypes.c_size_t(workspace.numel()),
                                                _stream(x)), "bnn_conv_f32_split_thr_ex")
    return (bits, y) if want_f32 else bits


def bwn_conv_thr(x, wbits, thr, C: int, stride: int, pad: int, want_f32: bool = False, workspace=None):
    """First layer with binarized weights: x [N][H][W][C] fp32, wbits [O][k][k][cw], thr [O] -> bits (and fp32 y)."""
    _dev(x, torch.float32, 4, "x"); _dev(wbits, _BITS, 4, "wbits"); _dev(thr, torch.float32, 1, "thr")
    N, H, W, C2 = x.shape
    O, k, _, cw = wbits.shape
    if C != C2 or cw != nwords(C):
        raise ValueError("channel mismatch")
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    bits = torch.empty((N, P, Q, nwords(O)), dtype=_BITS, device=x.device)
    y = torch.empty((N, P, Q, O), dtype=torch.float32, device=x.device) if want_f32 else None
    if workspace is None:
        workspace = torch.empty(max(int(load().bnn_bwn_workspace_bytes(C, O, k)), 16), dtype=torch.uint8, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().bnn_bwn_conv_thr(_ptr(x), _ptr(wbits), _ptr(thr), _ptr(y), _ptr(bits), N, H, W, C, O, k, int(stride), int(pad),
                                       _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(x)), "bnn_bwn_conv_thr")
    return (bits, y) if want_f32 else bits


def head_f32(bits, w, C: int, want_pooled: bool = False):
    """bits [N][H][W][cw] -> fp32 logits [N][J] = FC(sum-pool(+1/-1) / HW); w [J][C]."""
    _dev(bits, _BITS, 4, "bits"); _dev(w, torch.float32, 2, "w")
    N, H, W, cw = bits.shape
    J = w.shape[0]
    y = torch.empty((N, J), dtype=torch.float32, device=bits.device)
    pooled = torch.empty((N, C), dtype=torch.int32, device=bits.device) if want_pooled else None
    with torch.cuda.device(bits.device):
        _check(load().bnn_head_f32(_ptr(bits), _ptr(w), _ptr(y), _ptr(pooled), N, H * W, int(C), J, _stream(bits)), "bnn_head_f32")
    return (y, pooled) if want_pooled else y


class Net:
    """Layer-chained forward (bnn_net_*).  Keeps references to every weight tensor it borrows."""

    def __init__(self):
        self._h = ctypes.c_void_p()
        _check(load().bnn_net_create(ctypes.byref(self._h)), "bnn_net_create")
        self._keep = []
        self._ws = None
        self._out_kind = None
        self._out_cols = 0
        self.n_layers = 0

    def __del__(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            load().bnn_net_destroy(self._h)
            self._h = ctypes.c_void_p()

    def _added(self, *tensors):
        self._keep.extend(t for t in tensors if t is not None)
        self.n_layers += 1

    def input_u8(self, cols: int, thr: int):
        _check(load().bnn_net_input_u8(self._h, int(cols), int(thr)), "bnn_net_input_u8")
        self._in_dtype = torch.uint8
        self._added()

    def input_bits(self, cols: int):
        _check(load().bnn_net_input_bits(self._h, int(cols)), "bnn_net_input_bits")
        self._in_dtype = _BITS
        self._added()

    def input_conv_f32(self, w, thr, H: int, W: int, stride: int, pad: int):
        _dev(w, torch.float32, 4, "w"); _dev(thr, torch.float32, 1, "thr")
        O, k, _, C = w.shape
        _check(load().bnn_net_input_conv_f32(self._h, _ptr(w), _ptr(thr), int(H), int(W), C, O, k, int(stride), int(pad)),
               "bnn_net_input_conv_f32")
        self._in_dtype = torch.float32
        self._added(w, thr)

    def input_bwn_f32(self, wbits, thr, H: int, W: int, C: int, stride: int, pad: int):
        _dev(wbits, _BITS, 4, "wbits"); _dev(thr, torch.float32, 1, "thr")
        O, k, _, cw = wbits.shape
        if cw != nwords(C):
            raise ValueError("channel mismatch")
        _check(load().bnn_net_input_bwn_f32(self._h, _ptr(wbits), _ptr(thr), int(H), int(W), int(C), O, k, int(stride), int(pad)),
               "bnn_net_input_bwn_f32")
        self._in_dtype = torch.float32
        self._added(wbits, thr)

    def add_fc(self, W, thr, K: int):
        _dev(W, _BITS, 2, "W")
        if thr is not None:
            _dev(thr, torch.int32, 1, "thr")
        N = W.shape[0]
        if W.shape[1] != round_up(nwords(K), 4):
            raise ValueError("W rows must be ceil(K/32) words rounded up to a multiple of 4 (%d), got %d"
                             % (round_up(nwords(K), 4), W.shape[1]))
        _check(load().bnn_net_add_fc(self._h, _ptr(W), _ptr(thr), int(K), N), "bnn_net_add_fc")
        if thr is None:
            self._out_kind, self._out_cols = torch.int32, N
        self._added(W, thr)

    def add_conv(self, filt, thr, C: int, stride: int, pad: int, pad_mode: int = PAD_MINUS_ONE):
        _dev(filt, _BITS, 4, "filt"); _dev(thr, torch.int32, 1, "thr")
        O, k = filt.shape[0], filt.shape[1]
        _check(load().bnn_net_add_conv(self._h, _ptr(filt), _ptr(thr), int(C), O, k, int(stride), int(pad), int(pad_mode)),
               "bnn_net_add_conv")
        self._added(filt, thr)

    def add_pool(self, win: int, stride: int):
        _check(load().bnn_net_add_pool(self._h, int(win), int(stride)), "bnn_net_add_pool")
        self._added()

    def add_block(self, W1, thr1, W2, thr2, Wd, cin: int, cout: int, stride: int, pad_mode: int = PAD_MINUS_ONE):
        for t in (W1, W2):
            _dev(t, _BITS, 4, "W")
        _check(load().bnn_net_add_block(self._h, _ptr(W1), _ptr(thr1), _ptr(W2), _ptr(thr2), _ptr(Wd), int(cin), int(cout),
                                        int(stride), int(pad_mode)), "bnn_net_add_block")
        self._added(W1, thr1, W2, thr2, Wd)

    def add_head_f32(self, w):
        _dev(w, torch.float32, 2, "w")
        _check(load().bnn_net_add_head_f32(self._h, _ptr(w), w.shape[0]), "bnn_net_add_head_f32")
        self._out_kind, self._out_cols = torch.float32, w.shape[0]
        self._added(w)

    @classmethod
    def from_layers(cls, layers, in_hw: int, device="cuda"):
        """Builds a net from a list of layer dicts holding numpy arrays (the description the seeded
        generators and the CPU oracle use): conv_f32 first, then bconv / pool / block / fc."""
        import numpy as np

        def dev(a):
            a = np.ascontiguousarray(a)
            return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(device)

        net = cls()
        for L in layers:
            op = L["op"]
            if op == "conv_f32":
                net.input_conv_f32(dev(L["w"]), dev(L["thr"]), in_hw, in_hw, L["stride"], L["pad"])
            elif op == "bwn":
                net.input_bwn_f32(dev(L["W"]), dev(L["thr"]), in_hw, in_hw, L["C"], L["stride"], L["pad"])
            elif op == "bconv":
                net.add_conv(dev(L["W"]), dev(L["thr"]), L["C"], L["stride"], L["pad"])
            elif op == "pool":
                net.add_pool(L["win"], L["stride"])
            elif op == "block":
                net.add_block(dev(L["W1"]), dev(L["thr1"]), dev(L["W2"]), dev(L["thr2"]),
                              dev(L["Wd"]) if "Wd" in L else None, L["cin"], L["cout"], L["stride"])
            elif op == "fc":
                net.add_fc(dev(L["W"]), None if L["thr"] is None else dev(L["thr"]), L["K"])
            else:
                raise ValueError(op)
        return net

    def workspace_bytes(self, batch: int) -> int:
        n = ctypes.c_size_t()
        _check(load().bnn_net_workspace_bytes(self._h, int(batch), ctypes.byref(n)), "bnn_net_workspace_bytes")
        return n.value

    def forward(self, x, out=None, path: int = PATH_AUTO):
        _dev(x, self._in_dtype, None, "input")
        batch = x.shape[0]
        need = self.workspace_bytes(batch)
        if self._ws is None or self._ws.numel() < need or self._ws.device != x.device:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
        if out is None:
            out = torch.empty((batch, self._out_cols), dtype=self._out_kind, device=x.device)
        with torch.cuda.device(x.device):
            _check(load().bnn_net_forward(self._h, _ptr(x), _ptr(out), batch, _ptr(self._ws), ctypes.c_size_t(self._ws.numel()),
                                          int(path), _stream(x)), "bnn_net_forward")
        return out

    def forward_static(self, x, out=None, path: int = PATH_AUTO):
        """bnn_net_forward_static: the same forward on the library's fixed per-GPU workspace (no allocation inside
        the library; the output tensor must be passed in for a call that allocates nothing at all)."""
        _dev(x, self._in_dtype, None, "input")
        batch = x.shape[0]
        if out is None:
            out = torch.empty((batch, self._out_cols), dtype=self._out_kind, device=x.device)
        with torch.cuda.device(x.device):
            _check(load().bnn_net_forward_static(self._h, _ptr(x), _ptr(out), batch, int(path), _stream(x)),
                   "bnn_net_forward_static")
        return out

    def persistent_status(self, device=None) -> bool:
        """True if the last forward_persistent gave up at a barrier (its output is then undefined).  Waits for the
        current stream."""
        aborted = ctypes.c_int(-1)
        dev = self._ws.device if device is None else device
        with torch.cuda.device(dev):
            _check(load().bnn_net_persistent_status(self._h, ctypes.byref(aborted),
                                                    ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)),
                   "bnn_net_persistent_status")
        return aborted.value != 0

    def forward_persistent(self, x, out=None, no_sync: bool = False, give_up_at_once: bool = False, grid_cap: int = 0):
        """Same forward with every run of FC / 3x3 convolution / residual-block layers as one kernel launch.  no_sync
        skips the device-wide barriers (results undefined, for timing the barriers only); give_up_at_once makes every
        barrier wait time out at its first poll (results undefined, for testing the time-out report); grid_cap > 0
        bounds the number of workgroups."""
        _dev(x, self._in_dtype, None, "input")
        batch = x.shape[0]
        need = self.workspace_bytes(batch)
        if self._ws is None or self._ws.numel() < need or self._ws.device != x.device:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
        if out is None:
            out = torch.empty((batch, self._out_cols), dtype=self._out_kind, device=x.device)
        with torch.cuda.device(x.device):
            _check(load().bnn_net_forward_persistent(self._h, _ptr(x), _ptr(out), batch, _ptr(self._ws),
                                                     ctypes.c_size_t(self._ws.numel()),
                                                     (1 if no_sync else 0) | (2 if give_up_at_once else 0) | ((int(grid_cap) & 0xFFFF) << 8),
                                                     _stream(x)),
                   "bnn_net_forward_persistent")
        return out

    def layer_bits(self, layer: int):
        """Copy of the packed bits produced by `layer` in the last forward, as [rows][words]."""
        p = ctypes.c_void_p()
        rows = ctypes.c_int64()
        wpr = ctypes.c_int()
        _check(load().bnn_net_layer_bits(self._h, int(layer), ctypes.byref(p), ctypes.byref(rows), ctypes.byref(wpr)),
               "bnn_net_layer_bits")
        off = p.value - self._ws.data_ptr()
        n = rows.value * wpr.value * 4
        return self._ws[off:off + n].view(_BITS).view(rows.value, wpr.value).clone()
