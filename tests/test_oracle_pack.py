"""Pins for the oracle's nibble storage convention, pack/unpack, row sums and max-pool."""
import numpy as np
import pytest
import torch

from oracle import q4_oracle as o


def test_nibble_order_by_hand(golden):
    g = golden("handworked.txt")
    a = np.array(g["gemm_a"], dtype=np.uint8)
    b = np.array(g["gemm_b"], dtype=np.uint8)
    assert o.pack(a).tolist() == g["gemm_a_packed"]
    assert o.pack(b).tolist() == g["gemm_b_packed_kn"]
    assert o.pack(b, transpose=True).tolist() == g["gemm_b_packed_nk"]
    # element 0 -> low nibble, element 1 -> high nibble, odd tail -> high nibble 0
    assert o.pack(np.array([[0xA, 0x3, 0xF]], dtype=np.uint8)).tolist() == [[0x3A, 0x0F]]
    assert o.unpack(np.array([0x3A, 0x0F], dtype=np.uint8), 3).tolist() == [0xA, 0x3, 0xF]


@pytest.mark.parametrize("n", list(range(1, 66)))
def test_pack_unpack_round_trip(n):
    rng = np.random.default_rng(n)
    codes = rng.integers(0, 256, size=(3, n), dtype=np.uint8)   # upper bits must be ignored
    p = o.pack(codes)
    assert p.shape == (3, (n + 1) // 2)
    assert np.array_equal(o.unpack_rows(p, 3, n), codes & 15)
    if n % 2:
        assert np.all(p[:, -1] >> 4 == 0)
    # an independent NumPy statement of the same layout
    ref = np.zeros((3, (n + 1) // 2), dtype=np.uint8)
    for j in range(n):
        ref[:, j // 2] |= (codes[:, j] & 15) << (4 * (j % 2))
    assert np.array_equal(p, ref)


@pytest.mark.parametrize("rows,cols", [(1, 1), (2, 3), (5, 4), (7, 9), (16, 33)])
def test_pack_transpose(rows, cols):
    rng = np.random.default_rng(rows * 100 + cols)
    codes = rng.integers(0, 16, size=(rows, cols), dtype=np.uint8)
    assert np.array_equal(o.pack(codes, transpose=True), o.pack(np.ascontiguousarray(codes.T)))


def test_rowsum():
    rng = np.random.default_rng(5)
    for k in (1, 2, 9, 72, 145):
        codes = rng.integers(0, 16, size=(6, k), dtype=np.uint8)
        assert np.array_equal(o.rowsum(o.pack(codes), k), codes.astype(np.int64).sum(axis=1))
    # extremes: all fifteens
    assert o.rowsum(o.pack(np.full((1, 291), 15, np.uint8)), 291).tolist() == [291 * 15]


@pytest.mark.parametrize("N,H,W,C", [(1, 2, 2, 1), (2, 4, 6, 3), (1, 5, 7, 2), (3, 8, 8, 16)])
def test_maxpool_vs_torch(N, H, W, C):
    rng = np.random.default_rng(H * 10 + W)
    x = rng.integers(0, 16, size=(N, H, W, C), dtype=np.uint8)
    y = o.maxpool2x2(o.pack(x.reshape(1, -1)).reshape(-1), N, H, W, C)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2), 2, 2)
    ref = ref.permute(0, 2, 3, 1).numpy().astype(np.uint8)
    got = o.unpack(y, ref.size).reshape(ref.shape)
    assert np.array_equal(got, ref)


def test_maxpool_by_hand():
    # one 2x2 window per channel: max picks per-channel, not per-pixel
    x = np.array([[[[1, 9], [5, 2]], [[3, 4], [0, 15]]]], dtype=np.uint8)   # 1 x 2 x 2 x 2
    y = o.maxpool2x2(o.pack(x.reshape(1, -1)).reshape(-1), 1, 2, 2, 2)
    assert o.unpack(y, 2).tolist() == [5, 15]
