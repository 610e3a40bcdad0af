"""ctypes binding of the measured-peak probes (include/snn_peaks.h, libsnn_peaks.so).

Argument marshalling only.  Each call launches one probe kernel on torch's current stream; the
caller times it (HIP events on that stream) and divides the work stated in the header by the time.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsnn_peaks.so")
EXPORTS = ["snn_peak_copy", "snn_peak_fill", "snn_peak_read", "snn_peak_valu_xor_bcnt", "snn_peak_mfma_f4f6", "snn_peak_mfma_out_bytes",
           "snn_peak_swar_gather"]
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsnn_peaks.so is missing: run `python -m paper_2110_09195_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.snn_peak_copy.argtypes = [vp, vp, sz, vp]
        L.snn_peak_fill.argtypes = [vp, sz, ci, vp]
        L.snn_peak_read.argtypes = [vp, sz, ci, vp, vp]
        L.snn_peak_valu_xor_bcnt.argtypes = [vp, ci, ci, vp]
        L.snn_peak_mfma_f4f6.argtypes = [vp, ci, ci, ci, ci, vp]
        L.snn_peak_mfma_out_bytes.argtypes = [ci]
        L.snn_peak_mfma_out_bytes.restype = sz
        L.snn_peak_swar_gather.argtypes = [vp, vp, ci, ci, vp]
        for n in EXPORTS:
            if n != "snn_peak_mfma_out_bytes":
                getattr(L, n).restype = ci
        _lib = L
    return _lib


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with status %d" % (what, rc))


def copy(dst, src):
    _check(lib().snn_peak_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream()), "snn_peak_copy")


def fill(dst, nontemporal):
    _check(lib().snn_peak_fill(dst.data_ptr(), dst.numel() * dst.element_size(), int(nontemporal), _stream()), "snn_peak_fill")


READ_BLOCKS = 16384


def read(src, nontemporal, out):
    assert out.numel() >= READ_BLOCKS * 256
    _check(lib().snn_peak_read(src.data_ptr(), src.numel() * src.element_size(), int(nontemporal), out.data_ptr(), _stream()),
           "snn_peak_read")


def valu_xor_bcnt(out, iters, blocks):
    assert out.numel() * out.element_size() >= blocks * 1024
    _check(lib().snn_peak_valu_xor_bcnt(out.data_ptr(), iters, blocks, _stream()), "snn_peak_valu_xor_bcnt")
    return blocks * 256 * iters * 32          # lane-operations


def mfma_f4f6(out, shape, pattern, iters, blocks):
    assert out.numel() * out.element_size() >= lib().snn_peak_mfma_out_bytes(blocks)
    _check(lib().snn_peak_mfma_f4f6(out.data_ptr(), shape, pattern, iters, blocks, _stream()), "snn_peak_mfma_f4f6")
    return blocks * 4 * iters * 8             # matrix instructions


def swar_gather(out, idx, n_ci, blocks):
    assert idx.numel() >= n_ci * 64 + 48 and out.numel() >= blocks * 256
    _check(lib().snn_peak_swar_gather(out.data_ptr(), idx.data_ptr(), n_ci, blocks, _stream()), "snn_peak_swar_gather")
    return blocks * 256 * 4 * 64 * n_ci       # gather-adds
