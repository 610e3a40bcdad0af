"""Pins for the convolution oracle (CPU only).

Each test fixes the oracle to something outside it: a pure-Python brute force, a library
cross-correlation (torch CPU conv2d in float64), closed forms, or invariants the paper
states (Sec. 4.1 index end points, Sec. 4.5 / Fig. 6 sharing, 512-kernel subset == 1-bit).
"""
import numpy as np
import pytest
import torch

from tests import naive


def _rand_pm1(g, shape):
    return (g.integers(0, 2, size=shape) * 2 - 1).astype(np.int8)


def _weights_from_codes(codes):
    """[C_out][C_in] codes -> [C_out][C_in][3][3] via the paper's index assignment."""
    C_out, C_in = codes.shape
    w = np.zeros((C_out, C_in, 3, 3), dtype=np.int64)
    for co in range(C_out):
        for ci in range(C_in):
            w[co, ci] = naive.kernel_from_paper_index(int(codes[co, ci]) + 1)
    return w


# ---- Sec. 4.1: index assignment -------------------------------------------------------

def test_index_end_points(oracle):
    # golden: all -1 <-> paper index 1, all +1 <-> paper index 512
    rows = [l.split() for l in open(naive.GOLDEN_TABLES) if l.startswith("sec4.1")]
    ends = {r[1]: int(r[5]) for r in rows}
    assert (oracle.decode(ends["kernel_all_minus1"] - 1) == -1).all()
    assert (oracle.decode(ends["kernel_all_plus1"] - 1) == 1).all()


def test_decode_all_codes_match_binary_string(oracle):
    for code in range(512):
        assert (oracle.decode(code) == naive.kernel_from_paper_index(code + 1)).all()


def test_decode_is_msb_first_row_major(oracle):
    # code with only the most significant bit set: +1 at top-left only
    k = oracle.decode(0b100000000)
    assert k[0, 0] == 1 and k.sum() == 1 - 8
    # least significant bit: bottom-right
    k = oracle.decode(0b000000001)
    assert k[2, 2] == 1 and k.sum() == 1 - 8
    # bit 6 (third flattened element) is top-right, not left of the middle row
    k = oracle.decode(0b001000000)
    assert k[0, 2] == 1 and k.sum() == 1 - 8


# ---- brute force on tiny inputs --------------------------------------------------------

@pytest.mark.parametrize("stride", [1, 2])
def test_bin_conv_all_512_codes_brute_force(oracle, stride):
    g = np.random.default_rng(1)
    H, W = 4, 3
    xs = _rand_pm1(g, (1, 1, H, W))
    codes = np.arange(512, dtype=np.uint16).reshape(512, 1)   # every kernel as its own c_out
    alpha = np.ones(512, dtype=np.float32)
    S, Y = oracle.conv_bin(xs, codes, alpha, stride)
    ref = naive.conv3x3(xs.astype(np.int64), _weights_from_codes(codes), stride)
    assert S.shape == ref.shape
    assert (S == ref).all()
    assert (Y == ref.astype(np.float32)).all()


@pytest.mark.parametrize("stride,H,W", [(1, 4, 4), (2, 4, 4), (1, 1, 1), (2, 3, 4), (1, 2, 3), (2, 1, 4)])
def test_bin_conv_multichannel_brute_force(oracle, stride, H, W):
    g = np.random.default_rng(2 + H * 10 + W + stride)
    N, C_in, C_out = 2, 3, 4
    xs = _rand_pm1(g, (N, C_in, H, W))
    codes = g.integers(0, 512, size=(C_out, C_in)).astype(np.uint16)
    alpha = g.uniform(0.5, 1.5, size=C_out).astype(np.float32)
    S, Y = oracle.conv_bin(xs, codes, alpha, stride)
    ref = naive.conv3x3(xs.astype(np.int64), _weights_from_codes(codes), stride)
    assert (S == ref).all()
    # Y = float(S) * alpha, one fp32 multiply (numpy float32 multiply is that)
    assert (Y == ref.astype(np.float32) * alpha[None, :, None, None]).all()


@pytest.mark.parametrize("stride", [1, 2])
def test_f32_conv_brute_force(oracle, stride):
    g = np.random.default_rng(7)
    N, C_in, C_out, H, W = 2, 3, 3, 4, 3
    x = g.standard_normal((N, C_in, H, W)).astype(np.float32)
    codes = g.integers(0, 512, size=(C_out, C_in)).astype(np.uint16)
    alpha = g.uniform(0.5, 1.5, size=C_out).astype(np.float32)
    S, Y = oracle.conv_f32(x, codes, alpha, stride)
    ref = naive.conv3x3(x.astype(np.float64), _weights_from_codes(codes).astype(np.float64), stride)
    np.testing.assert_allclose(S, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(Y, ref * alpha[None, :, None, None].astype(np.float64), rtol=2e-7, atol=1e-7)


# ---- library routine: torch CPU conv2d (cross-correlation, zero padding) -----------------

def _torch_ref(x64, codes, stride):
    w = torch.from_numpy(_weights_from_codes(codes).astype(np.float64))
    return torch.nn.functional.conv2d(torch.from_numpy(x64), w, stride=stride, padding=1).numpy()


@pytest.mark.parametrize("stride,H,W,C_in,C_out", [(1, 14, 14, 32, 16), (2, 14, 14, 16, 24),
                                                   (1, 7, 9, 40, 8), (2, 9, 7, 5, 3), (1, 33, 35, 4, 4)])
def test_bin_conv_matches_library_cross_correlation(oracle, stride, H, W, C_in, C_out):
    g = np.random.default_rng(100 + H + W + C_in)
    xs = _rand_pm1(g, (3, C_in, H, W))
    codes = g.integers(0, 512, size=(C_out, C_in)).astype(np.uint16)
    alpha = np.ones(C_out, dtype=np.float32)
    S, Y = oracle.conv_bin(xs, codes, alpha, stride)
    ref = _torch_ref(xs.astype(np.float64), codes, stride)
    assert (S == ref.astype(np.int64)).all()       # small integers: the float64 conv is exact
    assert (Y == ref.astype(np.float32)).all()


@pytest.mark.parametrize("stride", [1, 2])
def test_f32_conv_matches_library_cross_correlation(oracle, stride):
    g = np.random.default_rng(11)
    x = g.standard_normal((4, 24, 8, 8)).astype(np.float32)
    codes = g.integers(0, 512, size=(16, 24)).astype(np.uint16)
    alpha = g.uniform(0.5, 1.5, size=16).astype(np.float32)
    S, Y = oracle.conv_f32(x, codes, alpha, stride)
    ref = _torch_ref(x.astype(np.float64), codes, stride)
    np.testing.assert_allclose(S, ref, rtol=0, atol=1e-11)
    np.testing.assert_allclose(Y, ref * alpha[None, :, None, None], rtol=2e-7, atol=1e-6)


def test_pins_discriminate_plausible_mistakes(oracle):
    """The inputs used above must be able to tell a flipped kernel (true convolution), a
    transposed kernel and an LSB-first bit order from the stated reading."""
    g = np.random.default_rng(5)
    xs = _rand_pm1(g, (2, 6, 6, 5))
    codes = g.integers(0, 512, size=(4, 6)).astype(np.uint16)
    S, _ = oracle.conv_bin(xs, codes, np.ones(4, np.float32), 1)
    w = _weights_from_codes(codes).astype(np.float64)
    x64 = torch.from_numpy(xs.astype(np.float64))

    def conv(wt):
        return torch.nn.functional.conv2d(x64, torch.from_numpy(np.ascontiguousarray(wt)), padding=1).numpy()

    assert (S == conv(w)).all()
    assert not (S == conv(w[:, :, ::-1, ::-1])).all()          # flipped: convolution proper
    assert not (S == conv(w.transpose(0, 1, 3, 2))).all()      # dy/dx swapped
    rev = np.array([[int(format(int(c), "09b")[::-1], 2) for c in row] for row in codes], dtype=np.uint16)
    assert not (S == conv(_weights_from_codes(rev).astype(np.float64))).all()   # LSB-first
    assert not (S == conv(-w)).all()                            # bit 1 <-> -1


# ---- closed forms ------------------------------------------------------------------------

@pytest.mark.parametrize("C_in", [1, 5, 32])
def test_all_plus_one_closed_form(oracle, C_in):
    H, W = 5, 6
    xs = np.ones((1, C_in, H, W), dtype=np.int8)
    codes = np.array([[511] * C_in, [0] * C_in], dtype=np.uint16)
    S, _ = oracle.conv_bin(xs, codes, np.ones(2, np.float32), 1)
    expect = np.full((H, W), 9 * C_in)
    expect[0, :] = expect[-1, :] = 6 * C_in
    expect[:, 0] = expect[:, -1] = 6 * C_in
    for r in (0, -1):
        for c in (0, -1):
            expect[r, c] = 4 * C_in
    assert (S[0, 0] == expect).all()
    assert (S[0, 1] == -expect).all()


def test_tap_isolation_gives_shifted_input(oracle):
    """(S_code - S_{code xor bit t}) / 2 is +-x shifted by tap t: pins tap order, bit order and
    that padding contributes zero."""
    g = np.random.default_rng(3)
    H, W = 5, 4
    xs = _rand_pm1(g, (1, 1, H, W))
    base = 0b101100110
    for t in range(9):
        dy, dx = divmod(t, 3)
        bit = 1 << (8 - t)
        codes = np.array([[base], [base ^ bit]], dtype=np.uint16)
        S, _ = oracle.conv_bin(xs, codes, np.ones(2, np.float32), 1)
        diff = (S[0, 0] - S[0, 1]) // 2
        sign_t = 1 if base & bit else -1
        shifted = np.zeros((H, W), dtype=np.int64)
        for h in range(H):
            for w in range(W):
                hh, ww = h + dy - 1, w + dx - 1
                if 0 <= hh < H and 0 <= ww < W:
                    shifted[h, w] = xs[0, 0, hh, ww]
        assert (diff == sign_t * shifted).all(), t


def test_parity_and_range(oracle):
    g = np.random.default_rng(4)
    C_in = 7
    xs = _rand_pm1(g, (2, C_in, 6, 6))
    codes = g.integers(0, 512, size=(5, C_in)).astype(np.uint16)
    S, _ = oracle.conv_bin(xs, codes, np.ones(5, np.float32), 1)
    assert np.abs(S).max() <= 9 * C_in
    assert ((S[:, :, 1:-1, 1:-1] - 9 * C_in) % 2 == 0).all()   # interior: parity of 9*C_in
    assert ((S[:, :, 0, 1:-1] - 6 * C_in) % 2 == 0).all()      # edge rows: 6 taps per channel


# ---- invariants the paper states ------------------------------------------------------------

@pytest.mark.parametrize("stride", [1, 2])
def test_two_stage_equals_direct_bin(oracle, stride):
    g = np.random.default_rng(20 + stride)
    K, C_in, C_out = 32, 12, 10
    xs = _rand_pm1(g, (2, C_in, 9, 7))
    codebook = np.sort(g.choice(512, size=K, replace=False)).astype(np.uint16)
    idx = g.integers(0, K, size=(C_out, C_in)).astype(np.uint16)
    alpha = g.uniform(0.5, 1.5, size=C_out).astype(np.float32)
    S1, Y1 = oracle.conv_bin(xs, oracle.expand(codebook, idx), alpha, stride)
    S2, Y2 = oracle.two_stage_bin(xs, codebook, idx, alpha, stride)
    assert (S1 == S2).all() and (Y1 == Y2).all()


@pytest.mark.parametrize("stride", [1, 2])
def test_two_stage_equals_direct_f32(oracle, stride):
    g = np.random.default_rng(23 + stride)
    K, C_in, C_out = 16, 12, 10
    x = g.standard_normal((2, C_in, 9, 8)).astype(np.float32)
    codebook = np.sort(g.choice(512, size=K, replace=False)).astype(np.uint16)
    idx = g.integers(0, K, size=(C_out, C_in)).astype(np.uint16)
    alpha = g.uniform(0.5, 1.5, size=C_out).astype(np.float32)
    S1, _ = oracle.conv_f32(x, oracle.expand(codebook, idx), alpha, stride)
    S2, _ = oracle.two_stage_f32(x, codebook, idx, alpha, stride)
    assert S1.shape == S2.shape == (2, C_out, (9 - 1) // stride + 1, (8 - 1) // stride + 1)
    rms = np.sqrt((S1 ** 2).mean())
    assert np.abs(S1 - S2).max() <= 1e-12 * rms * 100


def test_full_512_subset_is_the_one_bit_layer(oracle):
    """Sec. 4.1: a BNN kernel is one of 512; the subset of all 512 with idx = code is the BNN."""
    g = np.random.default_rng(30)
    C_in, C_out = 6, 5
    xs = _rand_pm1(g, (2, C_in, 6, 6))
    w9 = g.integers(0, 512, size=(C_out, C_in)).astype(np.uint16)
    alpha = g.uniform(0.5, 1.5, size=C_out).astype(np.float32)
    S_bnn, Y_bnn = oracle.conv_bin(xs, w9, alpha, 1)
    S_sub, Y_sub = oracle.two_stage_bin(xs, np.arange(512, dtype=np.uint16), w9, alpha, 1)
    assert (S_bnn == S_sub).all() and (Y_bnn == Y_sub).all()


def test_permuting_the_subset_changes_nothing_and_negation_negates(oracle):
    g = np.random.default_rng(31)
    K, C_in, C_out = 16, 8, 6
    xs = _rand_pm1(g, (1, C_in, 7, 7))
    codebook = g.choice(512, size=K, replace=False).astype(np.uint16)
    idx = g.integers(0, K, size=(C_out, C_in)).astype(np.uint16)
    alpha = np.ones(C_out, np.float32)
    S, _ = oracle.two_stage_bin(xs, codebook, idx, alpha, 1)
    perm = g.permutation(K)                       # new position j holds old entry perm[j]
    inv = np.argsort(perm)
    S_p, _ = oracle.two_stage_bin(xs, codebook[perm], inv[idx].astype(np.uint16), alpha, 1)
    assert (S == S_p).all()
    S_n, _ = oracle.two_stage_bin(xs, (511 - codebook).astype(np.uint16), idx, alpha, 1)
    assert (S_n == -S).all()


# ---- sign and packing ------------------------------------------------------------------------

def test_sign_reading(oracle):
    x = np.array([0.0, -0.0, 1e-30, -1e-30, np.nan, np.inf, -np.inf], dtype=np.float32)
    assert oracle.sign(x).tolist() == [1, 1, 1, -1, -1, 1, -1]


@pytest.mark.parametrize("W", [1, 7, 14, 32, 33, 56, 70])
def test_pack_rows_matches_packbits(oracle, W):
    g = np.random.default_rng(40 + W)
    x = g.standard_normal((2, 3, 4, W)).astype(np.float32)
    got = oracle.pack_rows(x)
    WW = (W + 31) // 32
    bits = np.zeros((2, 3, 4, WW * 32), dtype=np.uint8)
    bits[..., :W] = x >= 0
    ref = np.packbits(bits, axis=-1, bitorder="little").view(np.uint32).reshape(2, 3, 4, WW)
    assert (got == ref).all()


@pytest.mark.parametrize("C", [1, 16, 32, 40, 64, 100])
def test_pack_channels_matches_packbits(oracle, C):
    g = np.random.default_rng(50 + C)
    x = g.standard_normal((2, C, 3, 5)).astype(np.float32)
    got = oracle.pack_channels(x)
    CW = (C + 31) // 32
    bits = np.zeros((2, 3, 5, CW * 32), dtype=np.uint8)
    bits[..., :C] = (x >= 0).transpose(0, 2, 3, 1)
    ref = np.packbits(bits, axis=-1, bitorder="little").view(np.uint32).reshape(2, 3, 5, CW)
    assert (got == ref).all()


# ---- convolution + the next layer's sign (Alg. 1 forward, chained layers) ---------------------------

@pytest.mark.parametrize("stride,W", [(1, 9), (2, 37), (1, 33)])
def test_conv_sign_against_brute_force_threshold(oracle, stride, W):
    """bit = (S * alpha + beta >= 0): with alpha a power of two the fp32 product is exact, so the bit
    equals the integer comparison S * alpha >= -beta done in exact arithmetic (pure Python), for
    thresholds that sit exactly on attained values (the >= edge), between them, and for negative alpha
    (the comparison flips)."""
    from fractions import Fraction
    g = np.random.default_rng(300 + W)
    N, C_in, C_out, H = 2, 5, 6, 7
    xs = _rand_pm1(g, (N, C_in, H, W))
    codes = g.integers(0, 512, size=(C_out, C_in)).astype(np.uint16)
    alpha = np.array([0.5, -0.25, 2.0, 1.0, -1.0, 0.125], dtype=np.float32)
    beta = np.array([1.5, -0.75, 0.0, -3.0, 5.0, 0.0625], dtype=np.float32)       # exact in fp32, sums exact too
    S = naive.conv3x3(xs.astype(np.int64), _weights_from_codes(codes), stride)
    packed, pm1 = oracle.conv_sign(xs, codes, alpha, beta, stride)
    Ho, Wo = S.shape[2:]
    assert packed.shape == (N, C_out, Ho, (Wo + 31) // 32) and pm1.shape == S.shape
    for n in range(N):
        for co in range(C_out):
            for ho in range(Ho):
                for wo in range(Wo):
                    want = Fraction(int(S[n, co, ho, wo])) * Fraction(float(alpha[co])) + Fraction(float(beta[co])) >= 0
                    assert (int(packed[n, co, ho, wo // 32]) >> (wo % 32)) & 1 == int(want)
                    assert pm1[n, co, ho, wo] == (1 if want else -1)
    # unused high bits of a last word are zero
    if Wo % 32:
        assert (packed[..., -1] >> (Wo % 32) == 0).all()


def test_conv_sign_rounds_product_then_sum(oracle):
    """The product is rounded to fp32 before beta is added (no fused multiply-add).  Near 3 the fp32
    spacing is 2^-22; with alpha = 1 + 2^-23 and S = 3 the exact product 3 + 1.5 * 2^-22 is a tie and
    rounds to even, 3 + 2 * 2^-22.  beta = -(3 + 2 * 2^-22) then gives exactly 0 -> bit 1, where a
    fused multiply-add would see -0.5 * 2^-22 -> bit 0."""
    xs = np.ones((1, 1, 3, 3), dtype=np.int8)
    xs[0, 0, 0, :] = -1                                      # centre pixel: 6 - 3 with the all-ones kernel
    codes = np.array([[511]], dtype=np.uint16)
    alpha = np.array([1.0 + 2.0 ** -23], dtype=np.float32)
    assert float(alpha[0]) == 1.0 + 2.0 ** -23
    S, Y = oracle.conv_bin(xs, codes, alpha, 1)
    assert S[0, 0, 1, 1] == 3
    assert float(Y[0, 0, 1, 1]) == 3.0 + 2.0 ** -21
    beta = np.array([-(3.0 + 2.0 ** -21)], dtype=np.float32)
    assert float(beta[0]) == -(3.0 + 2.0 ** -21)
    packed, pm1 = oracle.conv_sign(xs, codes, alpha, beta, 1)
    assert pm1[0, 0, 1, 1] == 1 and (int(packed[0, 0, 1, 0]) >> 1) & 1 == 1
