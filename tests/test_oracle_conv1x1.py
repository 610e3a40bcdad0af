"""Pins for the oracle of the 1x1 extension (appendix, Table 5; CPU only)."""
import numpy as np
import pytest
import torch


def _rand_pm1(g, shape):
    return (g.integers(0, 2, size=shape) * 2 - 1).astype(np.int8)


def test_decode8_end_points_and_order(oracle):
    assert (oracle.decode8(0) == -1).all() and (oracle.decode8(255) == 1).all()
    assert oracle.decode8(0b10000000).tolist() == [1, -1, -1, -1, -1, -1, -1, -1]          # first element most significant
    assert oracle.decode8(0b00000001).tolist() == [-1, -1, -1, -1, -1, -1, -1, 1]


@pytest.mark.parametrize("stride", [1, 2])
def test_conv1x1_brute_force_and_library(oracle, stride):
    g = np.random.default_rng(80 + stride)
    N, G, C_out, H, W, K = 2, 3, 5, 4, 5, 7
    xs = _rand_pm1(g, (N, 8 * G, H, W))
    cb = g.permutation(256)[:K].astype(np.uint16)
    idx = g.integers(0, K, size=(C_out, G))
    alpha = g.uniform(0.5, 1.5, C_out).astype(np.float32)
    S, Y = oracle.conv1x1_bin(xs, cb, idx, alpha, stride)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    assert S.shape == (N, C_out, Ho, Wo)
    # pure Python, weight by weight from the binary string of the code
    for n in range(N):
        for co in range(C_out):
            for ho in range(Ho):
                for wo in range(Wo):
                    acc = 0
                    for gg in range(G):
                        bits = format(int(cb[idx[co, gg]]), "08b")
                        for j in range(8):
                            acc += (1 if bits[j] == "1" else -1) * int(xs[n, 8 * gg + j, ho * stride, wo * stride])
                    assert S[n, co, ho, wo] == acc
    # library 1x1 convolution in float64 on the decoded weights
    wmat = np.array([[1.0 if format(int(cb[idx[co, c // 8]]), "08b")[c % 8] == "1" else -1.0 for c in range(8 * G)]
                     for co in range(C_out)])
    ref = torch.nn.functional.conv2d(torch.from_numpy(xs.astype(np.float64)), torch.from_numpy(wmat)[:, :, None, None],
                                     stride=stride).numpy()
    assert (S == ref).all()
    assert (Y == (S.astype(np.float32) * alpha[None, :, None, None])).all()


def test_conv1x1_closed_forms(oracle):
    # all +1 activations and the all +1 member: S = C_in; the all -1 member: S = -C_in; parity of S = parity of C_in
    xs = np.ones((1, 16, 2, 2), dtype=np.int8)
    cb = np.array([255, 0, 0b10101010], dtype=np.uint16)
    S, _ = oracle.conv1x1_bin(xs, cb, np.array([[0, 0], [1, 1], [2, 2], [0, 1]]), np.ones(4, dtype=np.float32))
    assert (S[0, 0] == 16).all() and (S[0, 1] == -16).all() and (S[0, 2] == 0).all() and (S[0, 3] == 0).all()
    g = np.random.default_rng(5)
    xs = _rand_pm1(g, (2, 24, 3, 3))
    S, _ = oracle.conv1x1_bin(xs, g.permutation(256)[:16].astype(np.uint16), g.integers(0, 16, size=(6, 3)), np.ones(6, dtype=np.float32))
    assert (S % 2 == 0).all() and (np.abs(S) <= 24).all()
