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


def test_conv1x1_full_set_is_an_ordinary_binary_layer(oracle):
    # with all 256 vectors as the subset and idx = the code of sign(w), the layer is the 1-bit 1x1 layer
    g = np.random.default_rng(11)
    N, C_in, C_out, H, W = 2, 32, 6, 3, 4
    xs = _rand_pm1(g, (N, C_in, H, W))
    wsign = _rand_pm1(g, (C_out, C_in))
    codes = np.zeros((C_out, C_in // 8), dtype=np.int64)
    for j in range(8):
        codes = codes * 2 + (wsign[:, j::8] > 0)               # element j of every group, first element most significant
    S, _ = oracle.conv1x1_bin(xs, np.arange(256, dtype=np.uint16), codes, np.ones(C_out, dtype=np.float32))
    ref = np.einsum("oc,nchw->nohw", wsign.astype(np.int64), xs.astype(np.int64))
    assert (S == ref).all()


def test_conv1x1_single_element_isolation(oracle):
    # flipping element j of the vector of group gg changes S by -2 x[8 gg + j]: pins element order and channel grouping
    g = np.random.default_rng(12)
    G = 3
    xs = _rand_pm1(g, (1, 8 * G, 2, 3))
    one = np.ones(1, dtype=np.float32)
    for gg in range(G):
        for j in range(8):
            code = int(g.integers(0, 256)) | (1 << (7 - j))
            cb = np.array([code, code ^ (1 << (7 - j)), int(g.integers(0, 256))], dtype=np.uint16)
            base = np.full((1, G), 2)
            a, b = base.copy(), base.copy()
            a[0, gg], b[0, gg] = 0, 1
            Sa, _ = oracle.conv1x1_bin(xs, cb, a, one)
            Sb, _ = oracle.conv1x1_bin(xs, cb, b, one)
            assert ((Sa - Sb)[0, 0] == 2 * xs[0, 8 * gg + j].astype(np.int64)).all()


def test_conv1x1_inputs_tell_the_readings_apart(oracle):
    # the stated reading differs, on these inputs, from LSB-first element order and from strided channel grouping
    g = np.random.default_rng(13)
    G, C_out = 4, 5
    xs = _rand_pm1(g, (1, 8 * G, 3, 3))
    cb = g.permutation(256)[:8].astype(np.uint16)
    idx = g.integers(0, 8, size=(C_out, G))
    S, _ = oracle.conv1x1_bin(xs, cb, idx, np.ones(C_out, dtype=np.float32))
    w_lsb = np.array([[1 if (int(cb[idx[co, c // 8]]) >> (c % 8)) & 1 else -1 for c in range(8 * G)] for co in range(C_out)])
    w_strided = np.array([[1 if (int(cb[idx[co, c % G]]) >> (7 - c // G)) & 1 else -1 for c in range(8 * G)] for co in range(C_out)])
    for wrong in (w_lsb, w_strided):
        assert (np.einsum("oc,nchw->nohw", wrong, xs.astype(np.int64)) != S).any()
