"""Pins for the nearest-subset-member projection oracle (Eq. 1, Eq. 2, Eq. 5; CPU only)."""
import numpy as np

from tests import naive


def _bits_msb_first(w):
    """Eq. 1: sign(w) as a 9-bit code, first flattened element most significant."""
    code = 0
    for t in range(9):
        code = (code << 1) | (1 if w[t] >= 0 else 0)
    return code


def test_full_set_projection_is_sign(oracle):
    """Eq. 1: with all 512 kernels available the nearest kernel is sign(w)."""
    g = np.random.default_rng(0)
    w = g.standard_normal((5000, 9)).astype(np.float32)
    idx, score = oracle.project(w, np.arange(512, dtype=np.uint16))
    expect = np.array([_bits_msb_first(r) for r in w], dtype=np.uint16)
    assert (idx == expect).all()
    # the best inner product is the l1 norm
    np.testing.assert_allclose(score, np.abs(w).sum(axis=1), rtol=1e-6)


def test_subset_members_project_to_themselves(oracle):
    g = np.random.default_rng(1)
    codebook = g.choice(512, size=32, replace=False).astype(np.uint16)   # unsorted on purpose
    w = np.stack([naive.kernel_from_paper_index(int(c) + 1).reshape(9) for c in codebook]).astype(np.float32)
    idx, score = oracle.project(w, codebook)
    assert (idx == np.arange(32)).all()
    assert (score == 9.0).all()


def test_matches_float64_argmin_distance(oracle):
    """Eq. 2 as printed: arg min_k ||k - w||^2, brute force in float64."""
    g = np.random.default_rng(2)
    for K in (2, 16, 32, 64):
        codebook = g.choice(512, size=K, replace=False).astype(np.uint16)
        kernels = np.stack([naive.kernel_from_paper_index(int(c) + 1).reshape(9) for c in codebook]).astype(np.float64)
        w = g.standard_normal((4000, 9)).astype(np.float32)
        idx, _ = oracle.project(w, codebook)
        d = ((kernels[None, :, :] - w[:, None, :].astype(np.float64)) ** 2).sum(axis=2)
        ref = d.argmin(axis=1)
        differ = np.nonzero(idx != ref)[0]
        # any disagreement must be a float-level near tie between the two candidates
        for i in differ:
            assert abs(d[i, idx[i]] - d[i, ref[i]]) < 1e-5
        assert len(differ) <= 2


def test_lowest_index_wins_ties(oracle):
    codebook = np.array([7, 300, 511, 0], dtype=np.uint16)
    idx, score = oracle.project(np.zeros((3, 9), np.float32), codebook)
    assert (idx == 0).all() and (score == 0).all()
    # w with a single non-zero tap: every code with the right bit there ties
    w = np.zeros((1, 9), np.float32)
    w[0, 8] = 2.0                         # bottom-right tap wants +1: codes 7, 511 tie at +2
    idx, score = oracle.project(w, codebook)
    assert idx[0] == 0 and score[0] == 2.0
    w[0, 8] = -2.0                        # wants -1: codes 300 (even) and 0 tie
    idx, score = oracle.project(w, codebook)
    assert idx[0] == 1 and score[0] == 2.0


def test_scores_are_sequential_fp32_sums(oracle):
    """The score is built in fp32, taps 0..8 in order; a case where the order is visible."""
    w = np.array([[1e8, 1.0, -1e8, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0]], dtype=np.float32)
    codebook = np.array([511], dtype=np.uint16)
    _, score = oracle.project(w, codebook)
    acc = np.float32(0.0)
    for t in range(9):
        acc = np.float32(acc + w[0, t])
    assert score[0] == acc == np.float32(6.0)       # the first +1 is absorbed by 1e8
    assert float(np.sum(w.astype(np.float64))) == 7.0     # the exact sum differs


def test_k1_and_shapes(oracle):
    g = np.random.default_rng(3)
    w = g.standard_normal((4, 5, 3, 3)).astype(np.float32)
    idx, _ = oracle.project(w, np.array([123], dtype=np.uint16))
    assert idx.shape == (20,) and (idx == 0).all()
