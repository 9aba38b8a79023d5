"""Pins for the oracle GEMM: hand-worked values, brute force, the identity of Eq. (2),
extremes / overflow bound, and library routines.  None of these use the GPU."""
import itertools

import numpy as np
import pytest

from oracle import q4_oracle as o


def _py_gemm(a, za, b, zb):
    """Pure-Python triple loop over lists (brute force for tiny cases)."""
    M, K, N = len(a), len(a[0]), len(b[0])
    return [[sum((a[m][k] - za) * (b[k][n] - zb) for k in range(K)) for n in range(N)] for m in range(M)]


def test_handworked_2x2x2(golden):
    g = golden("handworked.txt")
    a = np.array(g["gemm_a_packed"], dtype=np.uint8)
    for layout, key in ((o.B_KN, "gemm_b_packed_kn"), (o.B_NK, "gemm_b_packed_nk")):
        b = np.array(g[key], dtype=np.uint8)
        assert o.gemm(a, g["gemm_za"], b, g["gemm_zb"], 2, 2, 2, layout).tolist() == g["gemm_c"]
        assert o.gemm_f64(a, g["gemm_za"], b, g["gemm_zb"], 2, 2, 2, layout).tolist() == g["gemm_c"]
    # zero points of zero give the raw code product
    b = np.array(g["gemm_b_packed_kn"], dtype=np.uint8)
    assert o.gemm(a, 0, b, 0, 2, 2, 2).tolist() == g["gemm_raw"]
    assert o.rowsum(a, 2).tolist() == g["gemm_rowsum_a"]
    assert o.rowsum(np.array(g["gemm_b_packed_nk"], dtype=np.uint8), 2).tolist() == g["gemm_colsum_b"]


def test_exhaustive_depth_two():
    """All 16^4 code tuples x all 16^2 zero points for M=N=1, K=2, against the closed form."""
    pairs = np.array(list(itertools.product(range(16), repeat=2)), dtype=np.uint8)   # 256 x 2
    A = o.pack(pairs)                                  # rows (a0, a1)
    B_nk = o.pack(pairs)                               # rows (b0, b1): N x K layout
    B_kn = o.pack(np.ascontiguousarray(pairs.T))       # 2 x 256: K x N layout
    a0 = pairs[:, 0].astype(np.int64)[:, None]
    a1 = pairs[:, 1].astype(np.int64)[:, None]
    b0 = pairs[:, 0].astype(np.int64)[None, :]
    b1 = pairs[:, 1].astype(np.int64)[None, :]
    for za in range(16):
        for zb in range(16):
            want = (a0 - za) * (b0 - zb) + (a1 - za) * (b1 - zb)
            assert np.array_equal(o.gemm(A, za, B_nk, zb, 256, 256, 2, o.B_NK), want)
            if (za + zb) % 5 == 0:
                assert np.array_equal(o.gemm(A, za, B_kn, zb, 256, 256, 2, o.B_KN), want)


def test_brute_force_tiny_shapes():
    """Non-square tiny shapes against a pure-Python loop: catches swapped or transposed indices."""
    rng = np.random.default_rng(11)
    for _ in range(150):
        M, N, K = (int(v) for v in rng.integers(1, 6, size=3))
        za, zb = (int(v) for v in rng.integers(0, 16, size=2))
        a = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
        b = rng.integers(0, 16, size=(K, N), dtype=np.uint8)
        want = _py_gemm(a.tolist(), za, b.tolist(), zb)
        assert o.gemm(o.pack(a), za, o.pack(b), zb, M, N, K, o.B_KN).tolist() == want
        assert o.gemm(o.pack(a), za, o.pack(b, transpose=True), zb, M, N, K, o.B_NK).tolist() == want


def test_exhaustive_2x2x2_reduced_alphabet():
    """2x2x2 products over the alphabet {0,1,7,8,15}^8 with za,zb in {0,7,8,15}: every position
    gets every extreme; checked against the four-term expansion of Eq. (2) in NumPy int64."""
    alpha = np.array([0, 1, 7, 8, 15], dtype=np.uint8)
    quads = np.array(list(itertools.product(alpha, repeat=4)), dtype=np.uint8)      # 625 x 4
    # A: rows are (a00 a01 | a10 a11) as 1250 rows of depth 2; B likewise as columns.
    A_codes = quads.reshape(-1, 2)                      # 1250 x 2
    B_codes = np.ascontiguousarray(quads.reshape(-1, 2).T)   # 2 x 1250
    A, B = o.pack(A_codes), o.pack(B_codes)
    raw = A_codes.astype(np.int64) @ B_codes.astype(np.int64)
    rs = A_codes.astype(np.int64).sum(1)[:, None]
    cs = B_codes.astype(np.int64).sum(0)[None, :]
    for za in (0, 7, 8, 15):
        for zb in (0, 7, 8, 15):
            want = raw - za * cs - zb * rs + 2 * za * zb
            assert np.array_equal(o.gemm(A, za, B, zb, 1250, 1250, 2), want)


@pytest.mark.parametrize("M,N,K", [(3, 5, 7), (17, 9, 33), (64, 32, 72), (40, 31, 145), (8, 24, 291)])
def test_identity_eq2_and_numpy_matmul(M, N, K):
    rng = np.random.default_rng(M * 1000 + N * 10 + K)
    za, zb = (int(v) for v in rng.integers(0, 16, size=2))
    a = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    b = rng.integers(0, 16, size=(K, N), dtype=np.uint8)
    A, Bkn, Bnk = o.pack(a), o.pack(b), o.pack(b, transpose=True)
    got = o.gemm(A, za, Bkn, zb, M, N, K, o.B_KN)
    a64, b64 = a.astype(np.int64), b.astype(np.int64)
    # library routine on the offset integers
    assert np.array_equal(got, (a64 - za) @ (b64 - zb))
    # Eq. (2), right-hand side: four terms computed separately
    four = a64 @ b64 - za * b64.sum(0)[None, :] - zb * a64.sum(1)[:, None] + K * za * zb
    assert np.array_equal(got, four)
    assert np.array_equal(o.gemm(A, za, Bnk, zb, M, N, K, o.B_NK), got)
    assert np.array_equal(o.gemm_f64(A, za, Bkn, zb, M, N, K, o.B_KN), got)
    assert np.array_equal(o.gemm_f64(A, za, Bnk, zb, M, N, K, o.B_NK), got)
    assert np.array_equal(o.gemm_rows(A, za, Bkn, zb, [M - 1, 0], N, K), got[[M - 1, 0]])


def test_extremes_at_depth_8192():
    K = 8192
    f = np.full((2, K), 15, np.uint8)
    z = np.zeros((2, K), np.uint8)
    P = o.pack
    assert np.all(o.gemm(P(f), 0, P(f), 0, 2, 2, K, o.B_NK) == 1843200)      # 8192 * 225
    assert np.all(o.gemm(P(z), 15, P(z), 15, 2, 2, K, o.B_NK) == 1843200)
    assert np.all(o.gemm(P(f), 0, P(z), 15, 2, 2, K, o.B_NK) == -1843200)
    assert np.all(o.gemm(P(np.full((2, K), 7, np.uint8)), 7, P(f), 3, 2, 2, K, o.B_NK) == 0)
    assert np.all(o.gemm(P(f), 3, P(np.full((2, K), 8, np.uint8)), 8, 2, 2, K, o.B_NK) == 0)


def test_int32_bound_is_the_analogue_of_the_depth_bound(golden):
    g = golden("paper_constants.txt")
    assert o.max_depth(2 ** 15 - 1, 4) == g["depth_bound_int16"]
    assert o.max_depth(2 ** 16 - 1, 4) == g["depth_bound_uint16"]
    assert o.max_channels(2 ** 15 - 1, 4, 1, 1) == g["channels_1x1"]
    assert o.max_channels(2 ** 15 - 1, 4, 3, 3) == g["channels_3x3"]
    assert o.max_channels(2 ** 15 - 1, 4, 5, 5) == g["channels_5x5"]
    kmax = o.max_depth(2 ** 31 - 1, 4)
    assert kmax == (2 ** 31 - 1) // g["max_product"] == 9544371
    # at the bound the all-fifteen product still fits; one more step does not
    row = o.pack(np.full((1, kmax + 1), 15, np.uint8))
    assert o.gemm(row, 0, row, 0, 1, 1, kmax, o.B_NK).tolist() == [[kmax * 225]]
    with pytest.raises(OverflowError):
        o.gemm(row, 0, row, 0, 1, 1, kmax + 1, o.B_NK)


def test_bad_arguments_are_rejected():
    a = np.zeros((2, 1), np.uint8)
    with pytest.raises(ValueError):
        o.gemm(a, 16, a, 0, 2, 2, 2)
    with pytest.raises(ValueError):
        o.gemm(a, 0, a, -1, 2, 2, 2)
    with pytest.raises(ValueError):
        o.gemm(a, 0, a, 0, 2, 2, 4)      # rows too short for K = 4


def test_gemm8_pins():
    """8-bit sibling: hand-worked value, NumPy int64 matmul, the four-term identity of Eq. (2), extremes."""
    # hand-worked: A = [[200, 10]], B_nk = [[0, 255]], za = 100, zb = 5: (100)(-5) + (-90)(250) = -500 - 22500
    assert o.gemm8(np.array([[200, 10]], np.uint8), 100, np.array([[0, 255]], np.uint8), 5).tolist() == [[-23000]]
    rng = np.random.default_rng(21)
    for M, N, K in ((3, 5, 7), (17, 9, 64), (33, 40, 200)):
        za, zb = (int(v) for v in rng.integers(0, 256, size=2))
        a = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        b = rng.integers(0, 256, size=(N, K), dtype=np.uint8)
        got = o.gemm8(a, za, b, zb)
        a64, b64 = a.astype(np.int64), b.astype(np.int64)
        assert np.array_equal(got, (a64 - za) @ (b64 - zb).T)
        four = a64 @ b64.T - za * b64.sum(1)[None, :] - zb * a64.sum(1)[:, None] + K * za * zb
        assert np.array_equal(got, four)
    K = 32768
    full, zero = np.full((1, K), 255, np.uint8), np.zeros((1, K), np.uint8)
    assert o.gemm8(full, 0, full, 0).tolist() == [[255 * 255 * K]]
    assert o.gemm8(full, 0, zero, 255).tolist() == [[-255 * 255 * K]]
