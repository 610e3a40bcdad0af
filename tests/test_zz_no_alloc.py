"""snn_subbit_conv2d_noalloc (the entry point for callers that cannot allocate) against
snn_subbit_conv2d and the oracle: called through the C ABI with raw pointers, two calls in a row on
the library's own buffer, the second on a smaller layer (which must not see the first one's tables)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2110_09195_amd import binding as B
from paper_2110_09195_amd import synth

pytestmark = pytest.mark.gpu


def _layer(seed, N, C_in, C_out, H, W, stride, K):
    g = synth.rng(77, seed)
    x = synth.activations(g, N, C_in, H, W)
    cb = synth.codebook(g, K)
    idx = synth.indices(g, C_out, C_in, K)
    alpha = synth.alpha(g, C_out)
    return x, cb, idx, alpha


def _dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


# the second layer of every pair is smaller in every dimension than the first
@pytest.mark.parametrize("first, second", [
    ((4, 96, 160, 14, 14, 1, 32), (2, 33, 40, 9, 7, 1, 32)),       # matrix-core kernel, then an odd, smaller layer
    ((2, 64, 64, 20, 20, 2, 16), (1, 8, 5, 6, 6, 1, 7)),           # stride 2, then a tiny layer with K = 7
    ((2, 40, 48, 10, 10, 1, 64), (2, 12, 16, 5, 5, 2, 64)),        # one input channel per matrix instruction (K = 64)
    ((1, 6, 10, 8, 8, 1, 512), (1, 3, 4, 4, 4, 1, 100)),           # the fallback kernel (K > 64)
])
def test_noalloc_matches_workspace_call_twice_in_a_row(oracle, first, second):
    L = B.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for seed, (N, C_in, C_out, H, W, stride, K) in enumerate((first, second)):
        print("case", (N, C_in, C_out, H, W, stride, K), flush=True)
        x, cb, idx, alpha = _layer(seed, N, C_in, C_out, H, W, stride, K)
        d = B.make_desc(N, C_in, C_out, H, W, stride, K, B.SNN_ACT_BIN_ROWS)
        xp = B.snn_pack_activations(_dev(x), B.SNN_ACT_BIN_ROWS)
        cb_d, idx_d, al_d = _dev(cb), _dev(idx), _dev(alpha)
        Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
        y_ws = B.snn_subbit_conv2d(d, xp, cb_d, idx_d, al_d)
        y = torch.full((N, C_out, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        rc = L.snn_subbit_conv2d_noalloc(ctypes.byref(d), ctypes.c_void_p(xp.data_ptr()), ctypes.c_void_p(cb_d.data_ptr()),
                                         ctypes.c_void_p(idx_d.data_ptr()), ctypes.c_void_p(al_d.data_ptr()),
                                         ctypes.c_void_p(y.data_ptr()), stream)
        assert rc == 0, B.status_string(rc)
        torch.cuda.synchronize()
        assert torch.equal(y, y_ws), "differs from snn_subbit_conv2d"
        _, Y = oracle.conv_bin(oracle.sign(x), oracle.expand(cb, idx), alpha, stride)
        assert (y.cpu().numpy() == Y).all(), "differs from the oracle"


def test_noalloc_refuses_layers_beyond_its_buffer():
    L = B.lib()
    # 2048 x 2048 kernels: the tables need more than the buffer holds
    d = B.make_desc(1, 2048, 2048, 4, 4, 1, 32, B.SNN_ACT_BIN_ROWS)
    assert B.snn_workspace_bytes(d, B.SNN_WS_SUBBIT) > 4 * 1024 * 1024
    t = torch.zeros(16, dtype=torch.int32, device="cuda")       # never read: the call returns before it enqueues anything
    p = ctypes.c_void_p(t.data_ptr())
    rc = L.snn_subbit_conv2d_noalloc(ctypes.byref(d), p, p, p, p, p, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == -3, B.status_string(rc)
