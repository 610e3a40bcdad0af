"""ctypes wrapper around oracle/snn_oracle.c (test infrastructure only).

All arrays are host numpy arrays.  Nothing here touches a GPU or the HIP library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "snn_oracle.c")
_LIB = os.path.join(_HERE, "libsnn_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc.  -ffp-contract=off keeps every fp32 operation a
    separately rounded IEEE operation (the scale multiply and the projection sums)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.snn_oracle_threads.restype = ctypes.c_int
        _lib.snn_oracle_out_size.restype = ctypes.c_int
        _lib.snn_oracle_two_stage_bin.restype = ctypes.c_int
        _lib.snn_oracle_two_stage_f32.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def threads():
    return int(_load().snn_oracle_threads())


def out_size(n, stride):
    return int(_load().snn_oracle_out_size(ctypes.c_int(n), ctypes.c_int(stride)))


def decode(code):
    """9-bit code -> (3,3) int8 array of +-1."""
    w = np.zeros(9, dtype=np.int8)
    _load().snn_oracle_decode(ctypes.c_uint16(int(code)), _p(w))
    return w.reshape(3, 3)


def sign(x):
    x = _c(x, np.float32)
    s = np.empty(x.shape, dtype=np.int8)
    _load().snn_oracle_sign(_p(x), _p(s), ctypes.c_int64(x.size))
    return s


def pack_rows(x):
    x = _c(x, np.float32)
    N, C, H, W = x.shape
    out = np.empty((N, C, H, (W + 31) // 32), dtype=np.uint32)
    _load().snn_oracle_pack_rows(_p(x), _p(out), N, C, H, W)
    return out


def pack_channels(x):
    x = _c(x, np.float32)
    N, C, H, W = x.shape
    out = np.empty((N, H, W, (C + 31) // 32), dtype=np.uint32)
    _load().snn_oracle_pack_channels(_p(x), _p(out), N, C, H, W)
    return out


def expand(codebook, idx):
    codebook = _c(codebook, np.uint16)
    idx = _c(idx, np.uint16)
    assert idx.size == 0 or int(idx.max()) < codebook.size
    codes = np.empty(idx.shape, dtype=np.uint16)
    _load().snn_oracle_expand(_p(codebook), _p(idx), ctypes.c_int64(idx.size), _p(codes))
    return codes


def _conv_args(x, codes, alpha, stride):
    N, C_in, H, W = x.shape
    codes = _c(codes, np.uint16)
    C_out = codes.shape[0]
    assert codes.shape == (C_out, C_in)
    assert codes.size == 0 or int(codes.max()) < 512
    alpha = _c(alpha, np.float32)
    assert alpha.shape == (C_out,)
    assert stride in (1, 2)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    return N, C_in, C_out, H, W, Ho, Wo, codes, alpha


def conv_bin(xs, codes, alpha, stride=1):
    """Direct convolution, +-1 activations.  xs: int8 NCHW in {+1,-1}; codes: [C_out][C_in]
    9-bit kernels.  Returns (S int32, Y float32), both [N][C_out][Ho][Wo]."""
    xs = _c(xs, np.int8)
    N, C_in, C_out, H, W, Ho, Wo, codes, alpha = _conv_args(xs, codes, alpha, stride)
    S = np.empty((N, C_out, Ho, Wo), dtype=np.int32)
    Y = np.empty((N, C_out, Ho, Wo), dtype=np.float32)
    _load().snn_oracle_conv_bin(_p(xs), N, C_in, C_out, H, W, stride, _p(codes), _p(alpha), _p(S), _p(Y))
    return S, Y


def conv_sign(xs, codes, alpha, beta, stride=1):
    """The convolution followed by the next layer's binarisation (Alg. 1 forward, sign(a^i), after
    the channel-wise affine alpha, beta): bit = (fl(fl(S * alpha) + beta) >= 0) in fp32, as packed
    rows uint32 [N][C_out][Ho][ceil(Wo/32)] and as the +-1 tensor the next conv_bin takes."""
    _, Y = conv_bin(xs, codes, alpha, stride)
    beta = _c(beta, np.float32)
    assert beta.shape == (Y.shape[1],)
    t = (Y + beta[None, :, None, None]).astype(np.float32)        # one fp32 rounding: Y and beta are fp32
    return pack_rows(t), sign(t)


def conv_f32(x, codes, alpha, stride=1):
    """Direct convolution, fp32 activations, float64 accumulation.
    Returns (S float64, Y float32)."""
    x = _c(x, np.float32)
    N, C_in, C_out, H, W, Ho, Wo, codes, alpha = _conv_args(x, codes, alpha, stride)
    S = np.empty((N, C_out, Ho, Wo), dtype=np.float64)
    Y = np.empty((N, C_out, Ho, Wo), dtype=np.float32)
    _load().snn_oracle_conv_f32(_p(x), N, C_in, C_out, H, W, stride, _p(codes), _p(alpha), _p(S), _p(Y))
    return S, Y


def _two_stage_args(x, codebook, idx, alpha, stride):
    N, C_in, H, W = x.shape
    codebook = _c(codebook, np.uint16)
    idx = _c(idx, np.uint16)
    C_out = idx.shape[0]
    assert idx.shape == (C_out, C_in)
    K = codebook.size
    assert idx.size == 0 or int(idx.max()) < K
    alpha = _c(alpha, np.float32)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    return N, C_in, C_out, H, W, Ho, Wo, K, codebook, idx, alpha


def two_stage_bin(xs, codebook, idx, alpha, stride=1):
    xs = _c(xs, np.int8)
    N, C_in, C_out, H, W, Ho, Wo, K, codebook, idx, alpha = _two_stage_args(xs, codebook, idx, alpha, stride)
    S = np.empty((N, C_out, Ho, Wo), dtype=np.int32)
    Y = np.empty((N, C_out, Ho, Wo), dtype=np.float32)
    rc = _load().snn_oracle_two_stage_bin(_p(xs), N, C_in, C_out, H, W, stride, _p(codebook), K,
                                          _p(idx), _p(alpha), _p(S), _p(Y))
    if rc != 0:
        raise MemoryError("oracle two-stage temporary")
    return S, Y


def two_stage_f32(x, codebook, idx, alpha, stride=1):
    x = _c(x, np.float32)
    N, C_in, C_out, H, W, Ho, Wo, K, codebook, idx, alpha = _two_stage_args(x, codebook, idx, alpha, stride)
    S = np.empty((N, C_out, Ho, Wo), dtype=np.float64)
    Y = np.empty((N, C_out, Ho, Wo), dtype=np.float32)
    rc = _load().snn_oracle_two_stage_f32(_p(x), N, C_in, C_out, H, W, stride, _p(codebook), K,
                                          _p(idx), _p(alpha), _p(S), _p(Y))
    if rc != 0:
        raise MemoryError("oracle two-stage temporary")
    return S, Y


def project(w, codebook):
    """Nearest subset member for every 3x3 kernel.  w: [..., 9] or [..., 3, 3] float32.
    Returns (idx uint16 [n], score float32 [n])."""
    w = _c(w, np.float32).reshape(-1, 9)
    codebook = _c(codebook, np.uint16)
    assert 1 <= codebook.size <= 512
    n = w.shape[0]
    idx = np.empty(n, dtype=np.uint16)
    score = np.empty(n, dtype=np.float32)
    _load().snn_oracle_project(_p(w), ctypes.c_int64(n), _p(codebook), int(codebook.size), _p(idx), _p(score))
    return idx, score


# ---- training side (Alg. 1 backward lines); plain numpy, float64 sums ---------------------------------

def project_backward(w, g_wbar, idx, K):
    """Eq. 3: the straight-through estimator, element by element: the gradient of the binarised kernel
    passes where -1 < w < 1 and is 0 elsewhere.  Backward of Eq. 5 (Alg. 1, update of p): the gradient
    of subset member k is the sum of the gradients of the binarised kernels that were assigned to it.
    w, g_wbar: [n][9] float32; idx: [n].  Returns (g_w float32 [n][9], g_p float64 [K][9])."""
    w = _c(w, np.float32).reshape(-1, 9)
    g = _c(g_wbar, np.float32).reshape(-1, 9)
    idx = np.asarray(idx).reshape(-1).astype(np.int64)
    assert w.shape == g.shape and idx.shape[0] == w.shape[0]
    assert idx.size == 0 or (0 <= idx.min() and idx.max() < K)
    inside = (w > np.float32(-1.0)) & (w < np.float32(1.0))
    g_w = np.where(inside, g, np.float32(0.0)).astype(np.float32)
    g_p = np.zeros((K, 9), dtype=np.float64)
    np.add.at(g_p, idx, g.astype(np.float64))
    return g_w, g_p


def subset_update(p, m, theta):
    """Eq. 4: m follows sign(p) where |p| > theta and keeps its value elsewhere; then the 9-bit code of
    every member (tap t at bit 8 - t, +1 -> 1) and, per member, whether an earlier member has the same
    code (Sec. 4.3: repeated members are to be replaced).  p: [K][9] float32, m: [K][9] in {+1, -1}.
    Returns (m' int8 [K][9], codes uint16 [K], dup uint8 [K])."""
    p = _c(p, np.float32).reshape(-1, 9)
    m = np.asarray(m, dtype=np.int8).reshape(-1, 9)
    assert p.shape == m.shape and theta >= 0
    follow = np.abs(p) > np.float32(theta)
    m2 = np.where(follow, np.where(p > 0, 1, -1), m).astype(np.int8)
    codes = np.zeros(p.shape[0], dtype=np.uint16)
    for k in range(p.shape[0]):
        for t in range(9):
            if m2[k, t] > 0:
                codes[k] |= np.uint16(1 << (8 - t))
    dup = np.zeros(p.shape[0], dtype=np.uint8)
    seen = set()
    for k in range(p.shape[0]):
        dup[k] = 1 if int(codes[k]) in seen else 0
        seen.add(int(codes[k]))
    return m2, codes, dup


def pack_indices(idx, tau):
    """Sec. 4.4 / Fig. 5: tau bits per kernel index.  Index i occupies bits [i * tau, (i + 1) * tau)
    of a little-endian bit stream of 32-bit words.  Returns uint32 [ceil(n * tau / 32)]."""
    idx = np.asarray(idx).reshape(-1).astype(np.uint32)
    assert 1 <= tau <= 9 and (idx.size == 0 or int(idx.max()) < (1 << tau))
    bits = ((idx[:, None] >> np.arange(tau, dtype=np.uint32)[None, :]) & 1).astype(np.uint8).reshape(-1)
    words = (bits.size + 31) // 32
    padded = np.zeros(words * 32, dtype=np.uint8)
    padded[:bits.size] = bits
    return np.packbits(padded, bitorder="little").view(np.uint32)


# ---- 1x1 layers (appendix: vectors of 8 input channels from a subset of {+-1}^8) ------------------------

def decode8(code):
    """8-bit code -> the +-1 vector: element j at bit 7 - j, bit 1 is +1 (the 3x3 reading applied to 8 elements)."""
    return np.array([1 if (int(code) >> (7 - j)) & 1 else -1 for j in range(8)], dtype=np.int64)


def project8(w, codebook8):
    """Nearest member of a subset of {+-1}^8 for each vector of 8 weights (appendix, Table 5; Eq. 2 /
    Eq. 5 with 8 elements): arg max_k of the inner product, accumulated in fp32 from 0 over elements
    0..7 in order (add or subtract), lowest index among equal scores.  Returns (idx uint16 [n],
    score float32 [n])."""
    w = _c(w, np.float32).reshape(-1, 8)
    codebook8 = _c(codebook8, np.uint16)
    K = codebook8.size
    signs = np.stack([decode8(int(c)) for c in codebook8]).astype(np.float32)        # [K][8], +-1
    score = np.zeros((w.shape[0], K), dtype=np.float32)
    for j in range(8):
        # fp32 add / subtract of w_j: multiplying by +-1 is exact, the sum rounds once
        score = (score + w[:, j:j + 1] * signs[None, :, j]).astype(np.float32)
    idx = np.argmax(score, axis=1)                                                     # first maximum
    return idx.astype(np.uint16), score[np.arange(w.shape[0]), idx]


def conv1x1_bin(xs, codebook8, idx, alpha, stride=1):
    """xs: int8 NCHW in {+1,-1}, C_in a multiple of 8; idx: [C_out][C_in / 8] into codebook8.
    The weight of (c_out, input channel 8 g + j) is element j of member idx[c_out][g]; the layer
    is the plain 1x1 convolution with those weights on the pixels (stride * h_out, stride * w_out).
    Returns (S int64, Y float32) [N][C_out][Ho][Wo], Y = (float)S * alpha."""
    xs = np.asarray(xs, dtype=np.int64)
    N, C_in, H, W = xs.shape
    idx = np.asarray(idx).astype(np.int64)
    C_out, G = idx.shape
    assert C_in == 8 * G and stride in (1, 2)
    members = np.stack([decode8(c) for c in np.asarray(codebook8).reshape(-1)])      # [K][8]
    wmat = members[idx].reshape(C_out, C_in)                                         # [C_out][G][8] -> [C_out][C_in]
    sub = xs[:, :, ::stride, ::stride]
    S = np.einsum("oc,nchw->nohw", wmat, sub)
    Y = (S.astype(np.float32) * _c(alpha, np.float32)[None, :, None, None]).astype(np.float32)
    return S, Y
