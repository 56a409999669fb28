"""GPU parity: bnn_bmm / bnn_bmm_thr through the C ABI against the CPU oracle, bit-exact."""
import ctypes

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


def run_case(bnn, orc, case, path, ref=None, ld_extra=0):
    A, B, tau = to_dev(case["A"]), to_dev(case["B"]), to_dev(case["tau"])
    K, N = case["K"], case["N"]
    ref = orc.bmm(case["A"], case["B"], K) if ref is None else ref
    C = host(bnn.bmm(A, B, K, path=path))
    assert np.array_equal(C, ref), "int32 mismatch: %d wrong" % int((C != ref).sum())
    ldcb = wl.round_up(wl.nwords(N), 4) + ld_extra
    bits = words(bnn.bmm_thr(A, B, tau, K, ldcb_w=ldcb, path=path))
    assert np.array_equal(bits, orc.threshold_pack(ref, case["tau"], ldb_w=ldcb)), "bit mismatch"


@pytest.mark.parametrize("pname,path", PATHS)
def test_cfg1_full(bnn, orc, pname, path):
    run_case(bnn, orc, wl.cfg1(), path)


SMALL = [(1, 1, 1), (1, 1, 32), (2, 3, 33), (7, 5, 127), (64, 64, 128), (65, 33, 129), (100, 130, 784),
         (8, 10, 1024), (257, 129, 4000), (300, 300, 96), (31, 513, 256), (129, 1000, 512), (40, 70, 2080)]


@pytest.mark.parametrize("pname,path", PATHS)
def test_ragged_shapes(bnn, orc, pname, path):
    for idx, (M, N, K) in enumerate(SMALL):
        print("shape", M, N, K, pname, flush=True)
        run_case(bnn, orc, wl.bmm_case(90, M, N, K, index0=10 * idx), path, ld_extra=4 if idx % 2 else 0)


# ragged shapes large enough to select each LDS-staged tile of the matrix-core path
STAGED = [(3000, 2500, 1000, "mfma_fp4_bmm_lds_wg128x128"), (5000, 5100, 1234, "mfma_fp4_bmm_xlds_wg256x256"),
          (131100, 50, 200, "mfma_fp4_bmm_lds_wg512x64"), (4097, 3001, 4100, "mfma_fp4_bmm_lds_wg256x128"),
          # the 256 x 256 tile with operands expanded into LDS: ragged edges on both sides, a last slab that is
          # half empty (K words = 4 mod 8), a single slab pair, and a short K that keeps the 256 x 128 kernel
          (4097, 3700, 1100, "mfma_fp4_bmm_xlds_wg256x256"), (3850, 4200, 1024, "mfma_fp4_bmm_xlds_wg256x256"),
          (4000, 4000, 800, "mfma_fp4_bmm_lds_wg256x128")]


@pytest.mark.parametrize("M,N,K,kernel", STAGED)
def test_ragged_shapes_staged_tiles(bnn, orc, M, N, K, kernel):
    assert bnn.bmm_kernel_name(M, N, K) == kernel
    case = wl.bmm_case(93, M, N, K, index0=M % 97)
    ref1 = orc.bmm(case["A"], case["B"], K, tier=1)
    for r0 in (0, M - 40):
        assert np.array_equal(orc.bmm_rows(case["A"], case["B"], K, r0, 40), ref1[r0:r0 + 40])
    run_case(bnn, orc, case, 0, ref=ref1, ld_extra=4)


@pytest.mark.parametrize("pname,path", PATHS)
def test_closed_forms_and_max_k(bnn, orc, pname, path):
    # K at the library's maximum: identical rows give +K, complemented rows -K (exactness of the
    # fp32 accumulation in the matrix-core path at its largest sum)
    K = 1 << 20
    M, N = 40, 33
    case = wl.bmm_case(91, M, N, K)
    case["B"][3] = case["A"][5]
    case["B"][4] = ~case["A"][6]
    C = host(bnn.bmm(to_dev(case["A"]), to_dev(case["B"]), K, path=path))
    assert C[5, 3] == K and C[6, 4] == -K
    ref = orc.bmm(case["A"], case["B"], K, tier=1)
    assert np.array_equal(C, ref)
    assert np.array_equal(orc.bmm_rows(case["A"], case["B"], K, 5, 2), C[5:7])


@pytest.mark.parametrize("n", [2048, 4096])
def test_sweep_squares_sampled(bnn, orc, n):
    # full output against the packed tier-1 oracle, 64 sampled rows against the naive tier-0 one
    case = wl.cfg2_case("sq%d" % n)
    ref1 = orc.bmm(case["A"], case["B"], n, tier=1)
    rows = [0, n - 64, n // 2 - 7]
    for r0 in rows:
        nr = 64 if r0 == n - 64 else 16
        assert np.array_equal(orc.bmm_rows(case["A"], case["B"], n, r0, nr), ref1[r0:r0 + nr])
    for pname, path in PATHS:
        print("n", n, pname, flush=True)
        run_case(bnn, orc, case, path, ref=ref1)


@pytest.mark.parametrize("name", ["fc8", "fc128", "fc1024"])
def test_sweep_fc(bnn, orc, name):
    case = wl.cfg2_case(name)
    ref1 = orc.bmm(case["A"], case["B"], case["K"], tier=1)
    nr = min(case["M"], 32)
    assert np.array_equal(orc.bmm_rows(case["A"], case["B"], case["K"], case["M"] - nr, nr), ref1[-nr:])
    for pname, path in PATHS:
        run_case(bnn, orc, case, path, ref=ref1)


@pytest.mark.parametrize("n", [8192, 16384])
def test_sweep_large_auto_path(bnn, orc, n):
    # the sizes bench.py times, in the launch configuration it uses (automatic path): the fused threshold bits
    # AND the whole int32 matrix against the packed tier-1 oracle, tier 1 itself against the naive tier 0 on
    # sampled rows
    case = wl.cfg2_case("sq%d" % n)
    A, B, tau = to_dev(case["A"]), to_dev(case["B"]), to_dev(case["tau"])
    bits = words(bnn.bmm_thr(A, B, tau, n))
    C = bnn.bmm(A, B, n)
    torch.cuda.synchronize()
    ref1 = orc.bmm(case["A"], case["B"], n, tier=1)
    assert np.array_equal(bits, orc.threshold_pack(ref1, case["tau"], ldb_w=bits.shape[1]))
    for r0 in (0, n // 3, n - 8):
        assert np.array_equal(orc.bmm_rows(case["A"], case["B"], n, r0, 8), ref1[r0:r0 + 8])
    step = 2048                                            # row chunks keep the host copies small
    for r0 in range(0, n, step):
        got = host(C[r0:r0 + step])
        assert np.array_equal(got, ref1[r0:r0 + step]), "int32 rows %d..%d: %d wrong" % (
            r0, r0 + step, int((got != ref1[r0:r0 + step]).sum()))


@pytest.mark.parametrize("n", [8192, 16384])
def test_sweep_large_k_panels(bnn, orc, n):
    # the same two sizes with both operands in K panels, as `bench.py --layout panels` runs them: the packed output (in
    # panels) and the whole int32 matrix against the tier-1 oracle (which the test above checks against tier 0)
    case = wl.cfg2_case("sq%d" % n)
    A, B, tau = to_dev(case["A"]), to_dev(case["B"]), to_dev(case["tau"])
    Ap, Bp = bnn.panels_from_rows(A, n), bnn.panels_from_rows(B, n)
    del A, B
    bits_p = words(bnn.bmm_thr_panels(Ap, Bp, tau, n))
    C = bnn.bmm_panels(Ap, Bp, n)
    torch.cuda.synchronize()
    ref1 = orc.bmm(case["A"], case["B"], n, tier=1)
    assert np.array_equal(bits_p, orc.panels(orc.threshold_pack(ref1, case["tau"], ldb_w=n // 32), n))
    step = 2048
    for r0 in range(0, n, step):
        got = host(C[r0:r0 + step])
        assert np.array_equal(got, ref1[r0:r0 + step]), "int32 rows %d..%d: %d wrong" % (
            r0, r0 + step, int((got != ref1[r0:r0 + step]).sum()))


@pytest.mark.parametrize("pname,path", [("auto", 0)] + PATHS)
def test_threshold_edge_values(bnn, orc, pname, path):
    # thresholds at and beyond the range of the sums, and at the ends of int32: columns whose B row equals or
    # complements an A row make the sums reach +K and -K exactly, so tau = K (bit 1), K + 1 (bit 0), -K (1),
    # -K - 1 (1) all decide a real equality; INT_MAX is never reached, INT_MIN always
    imin, imax = np.iinfo(np.int32).min, np.iinfo(np.int32).max
    for (M, N, K) in ((70, 96, 100), (130, 64, 1024), (33, 40, 4100), (300, 300, 777)):
        case = wl.bmm_case(94, M, N, K, index0=K % 91)
        edge = [K, K + 1, -K, -K - 1, K - 1, -K + 1, imin, imax, imin + 1, imax - 1, 0, 1, -1, 1 << 24, -(1 << 24), (1 << 24) + 1]
        for j, t in enumerate(edge):
            case["tau"][j] = t
            case["tau"][N - 1 - j] = t
            case["B"][j] = case["A"][j % M] if j % 2 == 0 else ~case["A"][j % M]
            case["B"][N - 1 - j] = ~case["A"][(j + 3) % M] if j % 2 == 0 else case["A"][(j + 3) % M]
        kw = wl.nwords(K)
        if K % 32:
            case["B"][:, kw - 1] &= np.uint32((1 << (K % 32)) - 1)          # complemented rows: pad bits back to 0
        case["B"][:, kw:] = 0
        ref = orc.bmm(case["A"], case["B"], K)
        assert (ref == K).any() and (ref == -K).any()
        print("edge thresholds", M, N, K, pname, flush=True)
        run_case(bnn, orc, case, path, ref=ref)


@pytest.mark.parametrize("M", [1, 7, 8, 9, 32, 33, 64, 65, 127, 128])
def test_skinny_rows(bnn, orc, M):
    # at most 128 rows: workgroups of 32 columns x all rows whose four waves split K.  K with one chunk, a ragged
    # last chunk (upper half-wave past the row's end), fewer chunks than waves, and many rounds per wave; N ragged
    assert bnn.bmm_kernel_name(M, 4096, 4096).startswith("mfma_fp4_bmm_skinny_m")
    assert bnn.bmm_kernel_name(129, 4096, 4096) != bnn.bmm_kernel_name(128, 4096, 4096)
    for idx, (N, K) in enumerate(((4096, 4096), (10, 1024), (1000, 784), (33, 100), (130, 257), (64, 5000), (96, 40000))):
        print("skinny", M, N, K, flush=True)
        case = wl.bmm_case(97, M, N, K, index0=(M * 7 + idx) % 89)
        ref = orc.bmm(case["A"], case["B"], K, tier=1)
        nr = min(M, 4)
        assert np.array_equal(orc.bmm_rows(case["A"], case["B"], K, M - nr, nr), ref[M - nr:])
        run_case(bnn, orc, case, 0, ref=ref, ld_extra=4 if idx % 2 else 0)


def test_skinny_max_k(bnn, orc):
    # K at the library's maximum through the skinny kernel (4096 chunks, 1024 rounds per wave): exact +-K
    K = 1 << 20
    for M in (8, 128):
        case = wl.bmm_case(98, M, 70, K, index0=M)
        case["B"][3] = case["A"][5]
        case["B"][4] = ~case["A"][6]
        ref = orc.bmm(case["A"], case["B"], K, tier=1)
        assert ref[5, 3] == K and ref[6, 4] == -K
        run_case(bnn, orc, case, 0, ref=ref)


def test_threshold_pack_and_packs(bnn, orc):
    rng = np.random.default_rng(5)
    for rows, cols, ld in [(1, 1, 1), (5, 77, 4), (130, 1024, 32), (33, 100, 8)]:
        X = rng.integers(-50, 51, size=(rows, cols)).astype(np.int32)
        tau = rng.integers(-20, 21, size=cols).astype(np.int32)
        got = words(bnn.threshold_pack(to_dev(X), to_dev(tau), ldb_w=ld))
        assert np.array_equal(got, orc.threshold_pack(X, tau, ldb_w=ld))
        x8 = rng.integers(0, 256, size=(rows, cols)).astype(np.uint8)
        assert np.array_equal(words(bnn.pack_u8(to_dev(x8), 127, ldb_w=ld)), orc.pack_u8(x8, 127, ldb_w=ld))
        xf = rng.normal(size=(rows, cols)).astype(np.float32)
        tf = rng.normal(size=cols).astype(np.float32)
        xf[0, 0] = tf[0]
        assert np.array_equal(words(bnn.pack_f32(to_dev(xf), to_dev(tf), ldb_w=ld)), orc.pack_f32(xf, tf, ldb_w=ld))
        bits = wl.random_bits(rng, rows, cols, ld)
        assert np.array_equal(host(bnn.unpack_i32(to_dev(bits), cols)), orc.unpack_pm1(bits, cols).astype(np.int32))


def test_error_codes(bnn):
    A = torch.zeros((4, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(bnn.BnnError) as e:
        bnn.bmm(A, A, 4 * 32 + 1)                 # K does not fit the leading dimension
    assert e.value.status == -1
    A6 = torch.zeros((4, 6), dtype=torch.int32, device="cuda")
    with pytest.raises(bnn.BnnError) as e:
        bnn.bmm(A6, A6, 100)                      # leading dimension not a multiple of 4 words
    assert e.value.status == -2
    with pytest.raises(bnn.BnnError) as e:
        bnn.bmm(A, A, 100, path=7)
    assert e.value.status == -1
    big = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    lib = bnn.load()
    assert lib.bnn_bmm(None, None, None, 1, 1, 1, 4, 4, 1, None) == -1
    p = __import__("ctypes").c_void_p(big.data_ptr())
    assert lib.bnn_bmm(p, p, p, 1, 1, (1 << 20) + 1, 1 << 16, 1 << 16, 1, None) == -3


@pytest.mark.parametrize("shape", [(9, 5, 70), (300, 200, 1000), (1024, 1024, 1024), (64, 129, 4097)])
def test_general_bmm_f32(bnn, orc, shape):
    # Sec. 7.2 "general" BMM: real-valued operands, binarized by sign on the way in, real-valued result
    M, N, K = shape
    rng = np.random.default_rng(sum(shape))
    A = rng.normal(size=(M, K)).astype(np.float32)
    B = rng.normal(size=(N, K)).astype(np.float32)
    A[0, 0] = 0.0
    B[N - 1, K - 1] = -0.0
    got = host(bnn.bmm_general_f32(to_dev(A), to_dev(B)))
    assert got.dtype == np.float32 and np.array_equal(got, orc.general_bmm_f32(A, B))
    zero = np.zeros(K, np.float32)
    assert np.array_equal(words(bnn.sign_pack_f32(to_dev(A))), orc.pack_f32(A, zero))


@pytest.mark.parametrize("shape", [(8, 4096, 4096), (128, 1000, 800), (300, 70, 1234), (1024, 1024, 1024), (2100, 2200, 512)])
def test_bmm_pretiled_weights(bnn, orc, shape):
    M, N, K = shape
    case = wl.bmm_case(96, M, N, K, index0=M % 89)
    Bt = bnn.tile_b(to_dev(case["B"]), K)
    assert np.array_equal(words(Bt), orc.tile_b(case["B"]))
    ref = orc.bmm(case["A"], case["B"], K, tier=1)
    assert np.array_equal(host(bnn.bmm_tiled(to_dev(case["A"]), Bt, N, K)), ref)
    bits = words(bnn.bmm_thr_tiled(to_dev(case["A"]), Bt, to_dev(case["tau"]), N, K))
    assert np.array_equal(bits, orc.threshold_pack(ref, case["tau"], ldb_w=wl.round_up(wl.nwords(N), 4)))


@pytest.mark.parametrize("shape", [(1, 1, 1), (300, 70, 1234), (257, 513, 256), (256, 256, 8192), (1000, 1500, 700), (2304, 2100, 2048),
                                   (4096, 4096, 4096), (40, 5000, 31)])
def test_bmm_k_panel_layout(bnn, orc, shape):
    # both operands in K panels, the packed output in panels too; conversions both ways against the layout's definition
    M, N, K = shape
    case = wl.bmm_case(97, M, N, K, index0=M % 83)
    Ap, Bp = bnn.panels_from_rows(to_dev(case["A"]), K), bnn.panels_from_rows(to_dev(case["B"]), K)
    assert np.array_equal(words(Ap), orc.panels(case["A"], K)) and np.array_equal(words(Bp), orc.panels(case["B"], K))
    back = words(bnn.rows_from_panels(Ap, K, ldx_w=case["A"].shape[1] + 4))
    assert np.array_equal(back[:, :case["A"].shape[1]], case["A"]) and not back[:, case["A"].shape[1]:].any()
    ref = orc.bmm(case["A"], case["B"], K, tier=1)
    assert np.array_equal(host(bnn.bmm_panels(Ap, Bp, K)), ref)
    tau = case["tau"].copy()
    edge = np.array([K, -K, K + 1, -K - 1, np.iinfo(np.int32).max, np.iinfo(np.int32).min], dtype=np.int64)
    tau[: min(N, 6)] = edge[: min(N, 6)].astype(np.int32)          # thresholds at and beyond the range of a sum
    bits_p = words(bnn.bmm_thr_panels(Ap, Bp, to_dev(tau), K))
    ref_bits = orc.threshold_pack(ref, tau, ldb_w=wl.nwords(N))
    assert np.array_equal(bits_p, orc.panels(ref_bits, N))
    # the output is the next product's row operand as it stands
    if M >= 256:
        nxt = wl.bmm_case(98, 8, 40, N)
        Wp = bnn.panels_from_rows(to_dev(nxt["B"]), N)
        assert np.array_equal(host(bnn.bmm_panels(to_dev(bits_p), Wp, N)), orc.bmm(ref_bits, nxt["B"], N, tier=1))


def test_k_panel_argument_errors(bnn):
    import torch
    X = torch.zeros((4, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(bnn.BnnError) as err:
        bnn.panels_from_rows(X, 300)                       # 300 bits do not fit rows of 8 words
    assert err.value.status == -1
    lib = bnn.load()
    P = torch.zeros((2, 4, 8), dtype=torch.int32, device="cuda")
    C = torch.zeros((4, 4), dtype=torch.int32, device="cuda")
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    assert lib.bnn_bmm_panels(ptr(P), ptr(P), None, 4, 4, 300, 4, None) == -1            # no output
    assert lib.bnn_bmm_panels(ptr(P), ptr(P), ptr(C), 4, 4, 300, 3, None) == -1          # ldc < N
    assert lib.bnn_bmm_panels(ctypes.c_void_p(P.data_ptr() + 4), ptr(P), ptr(C), 4, 4, 300, 4, None) == -2   # alignment
    assert lib.bnn_bmm_thr_panels(ptr(P), ptr(P), None, ptr(C), 4, 4, 300, None) == -1   # thresholds missing
    assert lib.bnn_bmm_panels(ptr(P), ptr(P), ptr(C), 4, 4, (1 << 20) + 1, 4, None) == -3   # K beyond the supported range


def test_probe_load_stride_runs(bnn):
    t = bnn.probe_load_stride(128, rows=256, iters=512)
    assert 1.0 < t < 1e5


def test_wide_leading_dimensions(bnn, orc):
    # rows of a much wider matrix (leading dimension 2^20 words): beyond the direct kernel's 32-bit lane offsets,
    # the call must still be exact (it takes the LDS-staged kernel)
    rng = np.random.default_rng(44)
    M, N, K, ld = 3, 5, 200, 1 << 20
    A = np.zeros((M, ld), np.uint32)
    B = np.zeros((N, ld), np.uint32)
    A[:, :8] = wl.random_bits(rng, (M,), K, ldw=8)
    B[:, :8] = wl.random_bits(rng, (N,), K, ldw=8)
    ref = orc.bmm(A[:, :8].copy(), B[:, :8].copy(), K)
    for path in (0, 2):
        assert np.array_equal(host(bnn.bmm(to_dev(A), to_dev(B), K, path=path)), ref)


@pytest.mark.parametrize("seed", [201, 202])
def test_random_shapes_all_paths(bnn, orc, seed):
    # 30 random shapes per seed (M, N around tile edges, K around word / 128-bit / chunk edges), int32 and bits out
    rng = np.random.default_rng(seed)
    for idx in range(30):
        M = int(rng.choice([1, 5, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 300]))
        N = int(rng.choice([1, 7, 31, 32, 33, 64, 65, 100, 128, 129, 260]))
        K = int(rng.choice([1, 31, 32, 33, 64, 100, 127, 128, 129, 255, 256, 257, 384, 500, 512, 1000, 1024, 1100, 4096, 5000]))
        print("bmm", M, N, K, flush=True)
        ld = wl.round_up(wl.nwords(K), 4)
        A = wl.random_bits(rng, (M,), K, ldw=ld)
        B = wl.random_bits(rng, (N,), K, ldw=ld)
        tau = wl.random_thresholds(rng, N, -40, 40)
        ref = orc.bmm(A, B, K)
        for path in (0, 1, 2):
            assert np.array_equal(host(bnn.bmm(to_dev(A), to_dev(B), K, path=path)), ref)
            bits = words(bnn.bmm_thr(to_dev(A), to_dev(B), to_dev(tau), K, path=path))
            assert np.array_equal(bits, orc.threshold_pack(ref, tau, ldb_w=bits.shape[1]))
