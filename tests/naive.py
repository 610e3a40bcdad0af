"""Deliberately naive second implementations used to pin the C oracle.

Pure Python / numpy, written independently of oracle/snn_oracle.c: the kernel of a code is
built from its binary string (as Sec. 4.1 describes the index assignment), and the
convolution works on an explicitly zero-padded copy of the input instead of testing bounds.
Only for tiny inputs.
"""
import os

import numpy as np

GOLDEN_TABLES = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_tables.txt")


def kernel_from_paper_index(index_1_based):
    """Sec. 4.1: flatten the 3x3 kernel, read it as a binary sequence, convert to decimal;
    all -1 is index 1 and all +1 is index 512."""
    bits = format(index_1_based - 1, "09b")            # first flattened element first
    flat = [1 if b == "1" else -1 for b in bits]
    return np.array(flat, dtype=np.int64).reshape(3, 3)


def conv3x3(x, kernels, stride):
    """x: [N][C_in][H][W]; kernels: [C_out][C_in][3][3]; zero padding 1; cross-correlation."""
    N, C_in, H, W = x.shape
    C_out = kernels.shape[0]
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    xp = np.zeros((N, C_in, H + 2, W + 2), dtype=x.dtype)
    xp[:, :, 1:H + 1, 1:W + 1] = x
    out = np.zeros((N, C_out, Ho, Wo), dtype=x.dtype)
    for n in range(N):
        for co in range(C_out):
            for ho in range(Ho):
                for wo in range(Wo):
                    window = xp[n, :, stride * ho:stride * ho + 3, stride * wo:stride * wo + 3]
                    out[n, co, ho, wo] = (window * kernels[co]).sum()
    return out
