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


# ---- projection of 8-vectors onto a subset of {+-1}^8 -------------------------------------------------

def test_project8_full_set_is_the_sign_pattern(oracle):
    # with all 256 members the nearest one is sign(w) (Eq. 1 applied to 8 elements) and the score is the 1-norm
    g = np.random.default_rng(21)
    w = g.standard_normal((500, 8)).astype(np.float32)
    idx, score = oracle.project8(w, np.arange(256, dtype=np.uint16))
    want = np.zeros(500, dtype=np.int64)
    for j in range(8):
        want = want * 2 + (w[:, j] >= 0)
    assert (idx == want).all()
    assert np.allclose(score, np.abs(w).sum(axis=1), rtol=1e-6)


def test_project8_members_project_to_themselves_and_brute_force(oracle):
    g = np.random.default_rng(22)
    cb = g.permutation(256)[:32].astype(np.uint16)
    members = np.array([[1.0 if (int(c) >> (7 - j)) & 1 else -1.0 for j in range(8)] for c in cb], dtype=np.float32)
    idx, score = oracle.project8(members, cb)
    assert (idx == np.arange(32)).all() and (score == 8.0).all()
    # float64 brute-force arg min of the squared distance agrees except at float-level near ties
    w = g.standard_normal((4000, 8)).astype(np.float32)
    idx, _ = oracle.project8(w, cb)
    d2 = ((w[:, None, :].astype(np.float64) - members[None, :, :].astype(np.float64)) ** 2).sum(axis=2)
    best = d2.argmin(axis=1)
    differ = np.nonzero(idx != best)[0]
    for i in differ:
        assert abs(d2[i, idx[i]] - d2[i, best[i]]) < 1e-5
    assert differ.size < 5


def test_project8_ties_go_to_the_lowest_index_and_order_matters(oracle):
    cb = np.array([0b11110000, 0b00001111, 0b11111111, 0b11110000], dtype=np.uint16)
    idx, _ = oracle.project8(np.zeros((1, 8), dtype=np.float32), cb)
    assert idx[0] == 0                                             # all scores 0
    idx, _ = oracle.project8(np.array([[1, 1, 1, 1, 0, 0, 0, 0]], dtype=np.float32), cb)
    assert idx[0] == 0                                             # members 0, 2 and 3 score 4: the first wins
    # sequential fp32 summation: (2^24 + 1) - 2^24 in this order loses the 1, the other order keeps it
    big = np.float32(2.0 ** 24)
    w = np.array([[big, 1.0, -big, 0, 0, 0, 0, 0], [big, -big, 1.0, 0, 0, 0, 0, 0]], dtype=np.float32)
    _, score = oracle.project8(w, np.array([255], dtype=np.uint16))
    assert score[0] == 0.0 and score[1] == 1.0
