"""Pins for the oracle's BMM, unpack and threshold (CPU only).

Every expected value here comes from something other than the oracle: pure-Python brute force on
+1/-1 lists built with an independent bit extraction, closed forms, the worked examples in
tests/golden/worked_examples.txt, and numpy's integer matmul on arrays unpacked with
numpy.unpackbits.
"""
import itertools
import os

import numpy as np
import pytest

import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.txt")


def np_unpack_pm1(words, nbits):
    """Independent unpack: numpy.unpackbits in little bit order on the little-endian bytes."""
    words = np.ascontiguousarray(words, dtype="<u4")
    b = np.unpackbits(words.view(np.uint8).reshape(words.shape[0], -1), axis=1, bitorder="little")
    return b[:, :nbits].astype(np.int32) * 2 - 1


def py_pm1(word_list, nbits):
    return [1 if (word_list[k // 32] >> (k % 32)) & 1 else -1 for k in range(nbits)]


def golden(kind):
    out = []
    with open(GOLD) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, args, exp = [s.strip() for s in line.split(";")]
            if k == kind:
                out.append((dict(a.split("=") for a in args.split()), int(exp)))
    return out


def test_golden_dot(orc):
    cases = golden("dot")
    assert len(cases) >= 5
    for args, exp in cases:
        n = int(args["n"])
        a = np.array([[int(t, 16) for t in args["a"].split(",")]], dtype=np.uint32)
        b = np.array([[int(t, 16) for t in args["b"].split(",")]], dtype=np.uint32)
        assert orc.bmm(a, b, n)[0, 0] == exp
        assert orc.bmm(a, b, n, tier=1)[0, 0] == exp


def test_golden_thr(orc):
    for args, exp in golden("thr"):
        bits = orc.threshold_pack(np.array([[int(args["v"])]], np.int32), np.array([int(args["tau"])], np.int32))
        assert int(bits[0, 0]) == exp


def test_unpack_convention(orc):
    # element k <-> word k//32, bit k%32 from the LSB; bit 1 = +1
    w = np.array([[0x00000001, 0x80000000, 0x2]], dtype=np.uint32)
    v = orc.unpack_pm1(w, 96)
    expect = -np.ones(96, dtype=np.int8)
    expect[0] = 1
    expect[63] = 1
    expect[65] = 1
    assert (v[0] == expect).all()
    rng = np.random.default_rng(7)
    w = rng.integers(0, 1 << 32, size=(5, 4), dtype=np.uint64).astype(np.uint32)
    assert (orc.unpack_pm1(w, 117) == np_unpack_pm1(w, 117)).all()


def test_exhaustive_small(orc):
    # all bit patterns for K <= 4 with M = N = 2, against Python integer arithmetic
    for K in (1, 2, 3, 4):
        pats = list(range(1 << K))
        for a0, a1 in itertools.product(pats, repeat=2):
            A = np.array([[a0], [a1]], dtype=np.uint32)
            for b0, b1 in itertools.product(pats, repeat=2) if K <= 3 else [(3, 12), (5, 10), (15, 0), (9, 6)]:
                B = np.array([[b0], [b1]], dtype=np.uint32)
                C = orc.bmm(A, B, K)
                C1 = orc.bmm(A, B, K, tier=1)
                for i, ai in enumerate((a0, a1)):
                    for j, bj in enumerate((b0, b1)):
                        ref = sum(x * y for x, y in zip(py_pm1([ai], K), py_pm1([bj], K)))
                        assert C[i, j] == ref and C1[i, j] == ref


@pytest.mark.parametrize("K", [1, 31, 32, 33, 63, 64, 65, 127, 129, 784])
def test_random_small_vs_python(orc, K):
    rng = np.random.default_rng(1000 + K)
    M, N = int(rng.integers(1, 8)), int(rng.integers(1, 8))
    ldw = wl.nwords(K) + int(rng.integers(0, 3))
    A = wl.random_bits(rng, M, K, ldw)
    B = wl.random_bits(rng, N, K, ldw)
    C = orc.bmm(A, B, K)
    for i in range(M):
        ai = py_pm1([int(x) for x in A[i]], K)
        for j in range(N):
            bj = py_pm1([int(x) for x in B[j]], K)
            assert C[i, j] == sum(x * y for x, y in zip(ai, bj))
    assert (orc.bmm(A, B, K, tier=1) == C).all()


@pytest.mark.parametrize("M,N,K", [(37, 29, 200), (64, 96, 1024), (130, 70, 784), (8, 10, 1024)])
def test_vs_numpy_matmul(orc, M, N, K):
    rng = np.random.default_rng(M * 7 + N)
    ldw = wl.round_up(wl.nwords(K), 4)
    A = wl.random_bits(rng, M, K, ldw)
    B = wl.random_bits(rng, N, K, ldw)
    ref = np_unpack_pm1(A, K) @ np_unpack_pm1(B, K).T       # note the transpose: B is N rows of K
    assert (orc.bmm(A, B, K) == ref).all()
    assert (orc.bmm(A, B, K, tier=1) == ref).all()
    assert (orc.bmm_rows(A, B, K, 3, 5) == ref[3:8]).all()
    # a non-square product would expose a transposed operand
    assert orc.bmm(A, B, K).shape == (M, N)


def test_closed_forms_and_invariants(orc):
    rng = np.random.default_rng(5)
    K, M = 333, 9
    ldw = wl.nwords(K)
    A = wl.random_bits(rng, M, K, ldw)
    mask = wl.random_bits(rng, 1, K, ldw) * 0 + np.uint32(0xFFFFFFFF)
    mask[..., -1] = np.uint32((1 << (K % 32)) - 1)
    # identical operands -> +K on the diagonal; complemented -> -K
    C = orc.bmm(A, A, K)
    assert (np.diag(C) == K).all()
    Ainv = (~A) & mask
    Cn = orc.bmm(A, Ainv, K)
    assert (np.diag(Cn) == -K).all()
    # complementing all of B negates C
    assert (Cn == -C).all()
    # symmetry C(A,B)^T = C(B,A)
    B = wl.random_bits(rng, 6, K, ldw)
    CAB, CBA = orc.bmm(A, B, K), orc.bmm(B, A, K)
    assert (CAB.T == CBA).all()
    # parity and bound
    assert ((CAB - K) % 2 == 0).all() and (np.abs(CAB) <= K).all()
    # a row of all +1 gives 2*popc(b) - K
    ones = mask.copy()
    pop = np.array([sum(bin(int(w)).count("1") for w in B[j]) for j in range(6)])
    assert (orc.bmm(ones, B, K)[0] == 2 * pop - K).all()
    # flipping one bit of A changes that row by exactly +-2 everywhere, nothing else
    A2 = A.copy()
    A2[4, 3] ^= np.uint32(1 << 17)
    d = orc.bmm(A2, B, K) - CAB
    assert (np.abs(d[4]) == 2).all() and (np.delete(d, 4, axis=0) == 0).all()


def test_statistics_cfg1(orc):
    # config 1 at full size: mean ~ 0, variance ~ K (sum of K independent +-1), tier 0 == tier 1
    case = wl.cfg1()
    C0 = orc.bmm(case["A"], case["B"], case["K"])
    C1 = orc.bmm(case["A"], case["B"], case["K"], tier=1)
    assert (C0 == C1).all()
    K = case["K"]
    assert abs(C0.mean()) < 4 * np.sqrt(K / C0.size) + 0.2
    assert abs(C0.var() / K - 1.0) < 0.02
    assert ((C0 - K) % 2 == 0).all()


def test_threshold_pack(orc):
    rng = np.random.default_rng(11)
    rows, cols = 13, 77
    X = rng.integers(-50, 51, size=(rows, cols)).astype(np.int32)
    tau = rng.integers(-20, 21, size=cols).astype(np.int32)
    bits = orc.threshold_pack(X, tau, ldb_w=4)
    assert bits.shape == (rows, 4)
    for r in range(rows):
        for c in range(128):
            got = (int(bits[r, c // 32]) >> (c % 32)) & 1
            exp = int(X[r, c] >= tau[c]) if c < cols else 0      # pad bits are written as 0
            assert got == exp
    # monotone: raising tau never sets more bits
    b2 = orc.threshold_pack(X, tau + 5, ldb_w=4)
    assert ((b2 & ~bits) == 0).all()
    # fraction of ones for a random product ~ 1 - Phi(tau / sqrt(K)) at tau = 0 -> about one half
    case = wl.bmm_case(9, 64, 256, 512)
    C = orc.bmm(case["A"], case["B"], 512)
    ones = np_unpack_pm1(orc.threshold_pack(C, np.zeros(256, np.int32)).reshape(64, -1), 256)
    assert abs((ones > 0).mean() - 0.52) < 0.05     # P(v >= 0) slightly above 1/2 since v = 0 counts


def test_pack_u8_f32(orc):
    rng = np.random.default_rng(3)
    x = rng.integers(0, 256, size=(5, 70)).astype(np.uint8)
    x[0, :4] = (126, 127, 128, 0)
    bits = orc.pack_u8(x, 127, ldb_w=4)
    ref = (x >= 127)
    assert (np_unpack_pm1(bits, 70) > 0).tolist() == ref.tolist()
    assert (np_unpack_pm1(bits, 128)[:, 70:] < 0).all()
    xf = rng.normal(size=(4, 3, 40)).astype(np.float32)
    tau = rng.normal(size=40).astype(np.float32)
    xf[0, 0, :3] = tau[:3]                     # equality counts as +1 (Eq. 1)
    bf = orc.pack_f32(xf, tau)
    assert (np_unpack_pm1(bf.reshape(12, -1), 40) > 0).tolist() == (xf >= tau).reshape(12, 40).tolist()


def test_bad_arguments(orc):
    A = np.zeros((2, 1), np.uint32)
    with pytest.raises(RuntimeError):
        orc.bmm(A, A, 40)          # K does not fit the leading dimension


def test_tile_b_layout_definition(orc):
    # element-by-element against the index formula, written with explicit loops
    rng = np.random.default_rng(11)
    for (N, K) in ((70, 256), (32, 128), (5, 640)):
        ldw = wl.round_up(wl.nwords(K), 4)
        B = wl.random_bits(rng, N, K, ldw)
        T = orc.tile_b(B).reshape(-1)
        upr = ldw // 4
        assert T.size == (N + 31) // 32 * 32 * ldw
        seen = np.zeros(T.size, bool)
        for r in range(N):
            for u in range(upr):
                d = ((r // 32) * upr + u) * 32 + r % 32
                assert (T[4 * d:4 * d + 4] == B[r, 4 * u:4 * u + 4]).all()
                seen[4 * d:4 * d + 4] = True
        assert (T[~seen] == 0).all()


def test_panels_layout_definition(orc):
    # element-by-element against the index formula of the header, written with explicit loops; bits past K are dropped
    rng = np.random.default_rng(12)
    for (rows, K, ldw) in ((70, 256, 8), (3, 300, 12), (33, 1000, 32), (5, 31, 4)):
        X = wl.random_bits(rng, rows, K, ldw)
        dirty = X.copy()
        if K % 32:
            dirty[:, K // 32] |= np.uint32(0xFFFFFFFF) << np.uint32(K % 32)     # junk past K must not travel
        dirty[:, wl.nwords(K):] = 0xDEADBEEF
        for src in (X, dirty):
            P = orc.panels(src, K)
            npan = (K + 255) // 256
            assert P.shape == (npan, rows, 8)
            flat = P.reshape(-1)
            seen = np.zeros(flat.size, bool)
            for r in range(rows):
                for w in range(wl.nwords(K)):
                    d = ((w // 8) * rows + r) * 8 + w % 8
                    assert flat[d] == X[r, w]
                    seen[d] = True
            assert (flat[~seen] == 0).all()
