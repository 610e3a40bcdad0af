"""Pins for the oracle's training-side steps (Alg. 1 backward lines; CPU only)."""
import numpy as np


def test_project_backward_closed_forms(oracle):
    g = np.random.default_rng(1)
    n, K = 300, 8
    w = (2.0 * g.standard_normal((n, 9))).astype(np.float32)
    gw = g.standard_normal((n, 9)).astype(np.float32)
    idx = g.integers(0, K, size=n)
    g_w, g_p = oracle.project_backward(w, gw, idx, K)
    # the member gradients add up to the total gradient (every kernel is assigned to exactly one member)
    assert np.allclose(g_p.sum(axis=0), gw.astype(np.float64).sum(axis=0), rtol=0, atol=1e-9)
    # all kernels on one member: that member gets everything
    _, g_one = oracle.project_backward(w, gw, np.full(n, 5), K)
    assert np.allclose(g_one[5], gw.astype(np.float64).sum(axis=0), atol=1e-9) and (np.delete(g_one, 5, axis=0) == 0).all()
    # brute force, member by member
    for k in range(K):
        want = np.zeros(9)
        for c in range(n):
            if idx[c] == k:
                want += gw[c].astype(np.float64)
        assert np.allclose(g_p[k], want, atol=1e-12)
    # Eq. 3 is element-wise on the open interval
    for c in range(n):
        for t in range(9):
            assert g_w[c, t] == (gw[c, t] if -1.0 < w[c, t] < 1.0 else 0.0)


def test_ste_interval_is_open_and_nan_blocks(oracle):
    w = np.array([[-1.0, 1.0, 0.99999994, -0.99999994, 0.0, -0.0, np.nan, np.inf, -np.inf]], dtype=np.float32)
    gw = np.arange(1, 10, dtype=np.float32).reshape(1, 9)
    g_w, _ = oracle.project_backward(w, gw, np.zeros(1, dtype=np.int64), 1)
    assert g_w.tolist() == [[0.0, 0.0, 3.0, 4.0, 5.0, 6.0, 0.0, 0.0, 0.0]]


def test_subset_update_hysteresis_codes_and_repeats(oracle):
    theta = 1e-3
    p = np.zeros((4, 9), dtype=np.float32)
    m = np.ones((4, 9), dtype=np.int8)
    m[1] = -1
    p[0, 0] = -0.5            # beyond the threshold: follows the sign of p
    p[0, 1] = -1e-3           # exactly theta: keeps its value (strict inequality)
    p[0, 2] = -0.0009         # inside the band: keeps its value
    p[1, :] = 0.002           # member 1 flips to all +1 ...
    p[2, 8] = -2.0
    p[3, 8] = -3.0            # ... members 2 and 3 become equal
    m2, codes, dup = oracle.subset_update(p, m, theta)
    assert m2[0].tolist() == [-1, 1, 1, 1, 1, 1, 1, 1, 1]
    assert (m2[1] == 1).all()
    assert codes.tolist() == [0b011111111, 0b111111111, 0b111111110, 0b111111110]
    assert dup.tolist() == [0, 0, 0, 1]
    # the code is the one the convolution oracle decodes back to the member
    for k in range(4):
        assert (oracle.decode(int(codes[k])).reshape(-1) == m2[k]).all()
    # theta = 0: every non-zero weight decides, zeros keep the memory
    m3, _, _ = oracle.subset_update(np.array([[0.0, -0.0, 1e-30, -1e-30, 1, -1, 0, 0, 0]], dtype=np.float32),
                                    -np.ones((1, 9), dtype=np.int8), 0.0)
    assert m3.tolist() == [[-1, -1, 1, -1, 1, -1, -1, -1, -1]]


def test_pack_indices_layout_and_ratio(oracle):
    """Sec. 4.4: tau bits per kernel, i.e. tau / 9 bit per weight.  A hand-written stream, the round
    trip through plain integer arithmetic, and the size."""
    # tau = 5: indices 1, 31, 0, 17, 8, 3, 30 -> bits 00001 11111 00000 10001 01000 00011 11110 (LSB first per index)
    idx = np.array([1, 31, 0, 17, 8, 3, 30], dtype=np.uint16)
    stream = sum(int(k) << (5 * i) for i, k in enumerate(idx))          # arbitrary-precision integer = the bit stream
    got = oracle.pack_indices(idx, 5)
    assert got.size == 2 and int(got[0]) == stream & 0xffffffff and int(got[1]) == stream >> 32
    g = np.random.default_rng(3)
    for tau in range(1, 10):
        n = int(g.integers(1, 400))
        idx = g.integers(0, 1 << tau, size=n).astype(np.uint16)
        packed = oracle.pack_indices(idx, tau)
        big = sum(int(w) << (32 * j) for j, w in enumerate(packed))
        assert [(big >> (tau * i)) & ((1 << tau) - 1) for i in range(n)] == idx.tolist()
        assert big >> (tau * n) == 0                                    # unused high bits are zero
        assert packed.size == (n * tau + 31) // 32
    # 512 x 512 kernels at tau = 5: 5 / 9 bit per weight against 1 bit for the 1-bit layer
    n = 512 * 512
    assert oracle.pack_indices(np.zeros(n, dtype=np.uint16), 5).size * 32 == n * 5
    assert abs(n * 5 / (n * 9) - 0.556) < 1e-3
