"""Closed-form operation and storage counts of Sec. 4.4 / Sec. 4.5.

Pure integer bookkeeping used by bench.py (work per layer) and by the tests that check the
layer lists in `synth` against the Bit-OPs and #Params columns the paper prints.
"""


def bnn_bit_ops(layer):
    """Sec. 4.5: a 1-bit 3x3 layer costs H*W*c_out*(c_in*3*3 + 1) bit-wise operations
    (H, W are the output resolution)."""
    return layer.H_out * layer.W_out * layer.C_out * (9 * layer.C_in + 1)


def snn_bit_ops(layer, K):
    """Sec. 4.5 as Tables 1-2 apply it: with a subset of K < c_out kernels the convolutions
    are shared (ratio K / c_out) and the index-gather/accumulate is charged half an operation
    per (c_out, c_in, pixel); with K >= c_out nothing is shared and the layer costs what
    the 1-bit layer costs.  The half-operation charge is inferred from the printed columns,
    which it reproduces to three digits; the text only states the ratio."""
    if K >= layer.C_out:
        return bnn_bit_ops(layer)
    hw = layer.H_out * layer.W_out
    return hw * K * (9 * layer.C_in + 1) + hw * layer.C_out * layer.C_in // 2


def storage_bits(layer, tau=None):
    """Sec. 4.4: 9 bits per kernel for a 1-bit layer; tau bits per kernel plus a subset of
    9 * 2^tau bits for a sub-bit layer."""
    kernels = layer.C_in * layer.C_out
    if tau is None:
        return 9 * kernels
    return tau * kernels + 9 * (1 << tau)


def stage1_responses(layer):
    """Stage 1 of Fig. 6: one response per (pixel, c_in, subset kernel)."""
    return layer.pixels * layer.C_in * layer.K


def stage2_gather_adds(layer):
    """Stage 2 of Fig. 6: one gather-add per (pixel, c_out, c_in)."""
    return layer.pixels * layer.C_out * layer.C_in
