"""Thin ctypes binding of the C ABI in include/snn.h.

Argument marshalling only: every function takes torch CUDA tensors (device memory) and passes
their pointers, sizes and the current HIP stream to the library entry point of the same name.
Nothing is computed here, and there is no fallback: if libsnn_hip.so has not been built the
first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsnn_hip.so")

SNN_OK = 0
SNN_ERR_INVALID_ARG = -1
SNN_ERR_UNSUPPORTED = -2
SNN_ERR_WORKSPACE = -3
SNN_ERR_LAUNCH = -4

SNN_ACT_BIN_ROWS = 0
SNN_ACT_BIN_CHANNELS = 1
SNN_ACT_F32 = 2

SNN_WS_SUBBIT = 0
SNN_WS_BNN = 1
SNN_WS_FORWARD = 2
SNN_WS_CONV1X1 = 3
SNN_WS_BNN_DENSE = 4

EXPORTS = ("snn_pack_activations", "snn_pack_activations_many", "snn_project_kernels", "snn_subbit_conv2d", "snn_subbit_conv2d_noalloc", "snn_subbit_forward",
           "snn_subbit_prepare", "snn_subbit_conv2d_prepared", "snn_packed_index_bytes", "snn_pack_indices",
           "snn_subbit_prepare_packed", "snn_subbit_conv1x1", "snn_subbit_conv1x1_prepare", "snn_subbit_conv1x1_prepared",
           "snn_project_vectors8",
           "snn_subbit_conv2d_sign", "snn_subbit_forward_sign", "snn_subbit_prepare_sign",
           "snn_subbit_conv2d_sign_prepared", "snn_subbit_project_prepare_many", "snn_subbit_conv2d_prepared_many",
           "snn_subbit_forward_many", "snn_project_backward",
           "snn_project_backward_workspace_bytes", "snn_subset_update", "snn_bnn_conv2d", "snn_bnn_prepare", "snn_bnn_conv2d_prepared", "snn_bnn_conv2d_dense",
           "snn_subbit_conv2d_dense", "snn_dense_prepare", "snn_dense_conv2d_prepared",
           "snn_dense_conv2d_sign_prepared",
           "snn_workspace_bytes", "snn_packed_bytes", "snn_status_string", "snn_subbit_slots_per_channel",
           "snn_set_tuning", "snn_get_tuning")


class snn_conv_desc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("C_in", ctypes.c_int32), ("C_out", ctypes.c_int32),
                ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("stride", ctypes.c_int32),
                ("K", ctypes.c_int32), ("act", ctypes.c_int32)]


class snn_layer_weights(ctypes.Structure):
    _fields_ = [("desc", snn_conv_desc), ("w", ctypes.c_void_p), ("codebook", ctypes.c_void_p), ("alpha", ctypes.c_void_p),
                ("beta", ctypes.c_void_p), ("idx_out", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                ("ws_bytes", ctypes.c_size_t)]


class snn_layer_io(ctypes.Structure):
    _fields_ = [("desc", snn_conv_desc), ("x_packed", ctypes.c_void_p), ("y_nchw", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class snn_pack_item(ctypes.Structure):
    _fields_ = [("x_nchw", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("N", ctypes.c_int32), ("C", ctypes.c_int32),
                ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("layout", ctypes.c_int32)]


class snn_layer_forward(ctypes.Structure):
    _fields_ = [("desc", snn_conv_desc), ("x_nchw", ctypes.c_void_p), ("w", ctypes.c_void_p), ("codebook", ctypes.c_void_p),
                ("alpha", ctypes.c_void_p), ("idx_out", ctypes.c_void_p), ("y_nchw", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class SnnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_string(status), status))


_lib = None


def lib():
    """Load libsnn_hip.so (built by `python -m paper_2110_09195_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library not built: %s is missing; run "
                               "`python -m paper_2110_09195_amd.build` (there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        dp = ctypes.POINTER(snn_conv_desc)
        L.snn_pack_activations.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.snn_pack_activations.restype = i32
        L.snn_project_kernels.argtypes = [vp, i64, vp, i32, vp, vp]
        L.snn_project_kernels.restype = i32
        L.snn_subbit_conv2d.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv2d.restype = i32
        L.snn_subbit_conv2d_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.snn_subbit_conv2d_noalloc.restype = i32
        L.snn_subbit_prepare.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_prepare.restype = i32
        L.snn_subbit_conv2d_prepared.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv2d_prepared.restype = i32
        L.snn_packed_index_bytes.argtypes = [i64, i32]
        L.snn_packed_index_bytes.restype = sz
        L.snn_pack_indices.argtypes = [vp, i64, i32, vp, vp]
        L.snn_pack_indices.restype = i32
        L.snn_subbit_prepare_packed.argtypes = [dp, vp, vp, i32, vp, vp, sz, vp]
        L.snn_subbit_prepare_packed.restype = i32
        L.snn_subbit_forward.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_forward.restype = i32
        L.snn_subbit_conv2d_sign.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv2d_sign.restype = i32
        L.snn_subbit_prepare_sign.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_prepare_sign.restype = i32
        L.snn_subbit_conv2d_sign_prepared.argtypes = [dp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv2d_sign_prepared.restype = i32
        L.snn_subbit_project_prepare_many.argtypes = [ctypes.POINTER(snn_layer_weights), i32, vp]
        L.snn_subbit_project_prepare_many.restype = i32
        L.snn_subbit_conv2d_prepared_many.argtypes = [ctypes.POINTER(snn_layer_io), i32, vp]
        L.snn_subbit_conv2d_prepared_many.restype = i32
        L.snn_pack_activations_many.argtypes = [ctypes.POINTER(snn_pack_item), i32, vp]
        L.snn_pack_activations_many.restype = i32
        L.snn_subbit_forward_many.argtypes = [ctypes.POINTER(snn_layer_forward), i32, vp]
        L.snn_subbit_forward_many.restype = i32
        L.snn_subbit_forward_sign.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_forward_sign.restype = i32
        L.snn_project_backward.argtypes = [vp, vp, vp, i64, i32, vp, vp, vp, sz, vp]
        L.snn_project_backward.restype = i32
        L.snn_project_backward_workspace_bytes.argtypes = [i64, i32]
        L.snn_project_backward_workspace_bytes.restype = sz
        L.snn_subset_update.argtypes = [vp, vp, ctypes.c_float, i32, vp, vp, vp]
        L.snn_subset_update.restype = i32
        L.snn_subbit_conv1x1.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv1x1.restype = i32
        L.snn_subbit_conv1x1_prepare.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv1x1_prepare.restype = i32
        L.snn_subbit_conv1x1_prepared.argtypes = [dp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv1x1_prepared.restype = i32
        L.snn_bnn_conv2d.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_bnn_conv2d.restype = i32
        L.snn_bnn_prepare.argtypes = [dp, vp, vp, sz, vp]
        L.snn_bnn_prepare.restype = i32
        L.snn_bnn_conv2d_prepared.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.snn_bnn_conv2d_prepared.restype = i32
        L.snn_bnn_conv2d_dense.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_bnn_conv2d_dense.restype = i32
        L.snn_subbit_conv2d_dense.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_subbit_conv2d_dense.restype = i32
        L.snn_dense_prepare.argtypes = [dp, vp, vp, vp, sz, vp]
        L.snn_dense_prepare.restype = i32
        L.snn_dense_conv2d_prepared.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.snn_dense_conv2d_prepared.restype = i32
        L.snn_project_vectors8.argtypes = [vp, ctypes.c_int64, vp, ctypes.c_int, vp, vp]
        L.snn_project_vectors8.restype = i32
        L.snn_dense_conv2d_sign_prepared.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.snn_dense_conv2d_sign_prepared.restype = i32
        L.snn_workspace_bytes.argtypes = [dp, i32]
        L.snn_workspace_bytes.restype = sz
        L.snn_packed_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.snn_packed_bytes.restype = sz
        L.snn_status_string.argtypes = [i32]
        L.snn_status_string.restype = ctypes.c_char_p
        L.snn_subbit_slots_per_channel.argtypes = [dp]
        L.snn_subbit_slots_per_channel.restype = i32
        L.snn_set_tuning.argtypes = [i32, i32]
        L.snn_set_tuning.restype = i32
        L.snn_get_tuning.argtypes = [i32]
        L.snn_get_tuning.restype = i32
        _lib = L
    return _lib


def status_string(status):
    return lib().snn_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != SNN_OK:
        raise SnnError(status, where)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))
    return t


def make_desc(N, C_in, C_out, H, W, stride=1, K=32, act=SNN_ACT_BIN_ROWS):
    return snn_conv_desc(N, C_in, C_out, H, W, stride, K, act)


def out_hw(desc):
    return (desc.H - 1) // desc.stride + 1, (desc.W - 1) // desc.stride + 1


def snn_packed_bytes(N, C, H, W, layout):
    return int(lib().snn_packed_bytes(N, C, H, W, layout))


SNN_TUNE_AUTO = -1
(SNN_TUNE_SUBBIT_MFMA, SNN_TUNE_MFMA_TILE, SNN_TUNE_MFMA_KS, SNN_TUNE_MFMA_STAGE, SNN_TUNE_MFMA_QUAD, SNN_TUNE_STACK,
 SNN_TUNE_BNN_REGS, SNN_TUNE_DENSE_TILE, SNN_TUNE_F32_WAVES) = range(9)
SNN_TUNE_COUNT = 9


def snn_set_tuning(knob, value):
    _check(lib().snn_set_tuning(knob, value), "snn_set_tuning")


def snn_get_tuning(knob):
    return int(lib().snn_get_tuning(knob))


def snn_subbit_slots_per_channel(desc):
    r = int(lib().snn_subbit_slots_per_channel(ctypes.byref(desc)))
    if r < 0:
        _check(r, "snn_subbit_slots_per_channel")
    return r


def snn_workspace_bytes(desc, which):
    return int(lib().snn_workspace_bytes(ctypes.byref(desc), which))


def alloc_workspace(desc, which, device="cuda"):
    n = snn_workspace_bytes(desc, which)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def snn_pack_activations(x, layout, out=None):
    """x: float32 [N][C][H][W] on the GPU -> packed int32 tensor (flat words) in `layout`."""
    _dev(x, torch.float32, "x")
    N, C, H, W = x.shape
    nbytes = snn_packed_bytes(N, C, H, W, layout)
    if out is None:
        out = torch.empty(nbytes // 4, dtype=torch.int32, device=x.device)
    _dev(out, torch.int32, "out")
    if out.numel() * 4 < nbytes:
        raise ValueError("packed buffer too small")
    _check(lib().snn_pack_activations(_ptr(x), _ptr(out), N, C, H, W, layout, _stream()), "snn_pack_activations")
    return out


def pack_item_array(items):
    """items: list of (x float32 [N][C][H][W], out packed int32 tensor, layout) -> a ctypes array for
    snn_pack_activations_many; build it once and reuse it (the tensors must stay alive)."""
    arr = (snn_pack_item * len(items))()
    for i, (x, out, layout) in enumerate(items):
        _dev(x, torch.float32, "x")
        _dev(out, torch.int32, "out")
        N, C, H, W = x.shape
        if out.numel() * 4 != snn_packed_bytes(N, C, H, W, layout):
            raise ValueError("out has the wrong size")
        arr[i].x_nchw = x.data_ptr()
        arr[i].packed = out.data_ptr()
        arr[i].N, arr[i].C, arr[i].H, arr[i].W = N, C, H, W
        arr[i].layout = layout
    return arr


def snn_pack_activations_many(arr):
    _check(lib().snn_pack_activations_many(arr, len(arr), _stream()), "snn_pack_activations_many")


def snn_project_kernels(w, codebook, out=None):
    """w: float32 [n][9]; codebook: int16 [K] (9-bit codes) -> int16 [n] indices."""
    _dev(w, torch.float32, "w")
    _dev(codebook, torch.int16, "codebook")
    n = w.numel() // 9
    if out is None:
        out = torch.empty(n, dtype=torch.int16, device=w.device)
    _dev(out, torch.int16, "out")
    _check(lib().snn_project_kernels(_ptr(w), n, _ptr(codebook), codebook.numel(), _ptr(out), _stream()),
           "snn_project_kernels")
    return out


def _conv_out(desc, y, device):
    Ho, Wo = out_hw(desc)
    if y is None:
        y = torch.empty((desc.N, desc.C_out, Ho, Wo), dtype=torch.float32, device=device)
    _dev(y, torch.float32, "y")
    if y.numel() != desc.N * desc.C_out * Ho * Wo:
        raise ValueError("y has the wrong size")
    return y


def snn_subbit_conv2d(desc, x, codebook, idx, alpha, y=None, workspace=None):
    """x: packed int32 (rows layout) or float32 NCHW per desc.act; codebook int16 [K];
    idx int16 [C_out][C_in]; alpha float32 [C_out] -> y float32 [N][C_out][Ho][Wo]."""
    _dev(codebook, torch.int16, "codebook")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_SUBBIT, x.device)
    _check(lib().snn_subbit_conv2d(ctypes.byref(desc), _ptr(x), _ptr(codebook), _ptr(idx), _ptr(alpha), _ptr(y),
                                   _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_conv2d")
    return y


def snn_subbit_conv2d_noalloc(desc, x, codebook, idx, alpha, y):
    """snn_subbit_conv2d without a workspace (the library's own per-GPU buffer); `y` must be given:
    neither the call nor this wrapper allocates."""
    _dev(codebook, torch.int16, "codebook")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    _dev(y, torch.float32, "y")
    if y.numel() != desc.N * desc.C_out * ((desc.H - 1) // desc.stride + 1) * ((desc.W - 1) // desc.stride + 1):
        raise ValueError("y has the wrong size")
    _check(lib().snn_subbit_conv2d_noalloc(ctypes.byref(desc), _ptr(x), _ptr(codebook), _ptr(idx), _ptr(alpha), _ptr(y),
                                           _stream()), "snn_subbit_conv2d_noalloc")
    return y


def snn_subbit_prepare(desc, codebook, idx, alpha, workspace=None):
    """Weights -> tables in `workspace` (returned); then any number of snn_subbit_conv2d_prepared calls."""
    _dev(codebook, torch.int16, "codebook")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_SUBBIT, codebook.device)
    _check(lib().snn_subbit_prepare(ctypes.byref(desc), _ptr(codebook), _ptr(idx), _ptr(alpha), _ptr(workspace),
                                    workspace.numel(), _stream()), "snn_subbit_prepare")
    return workspace


def snn_pack_indices(idx, tau):
    """idx int16 [n] -> int32 words holding tau bits per index."""
    _dev(idx, torch.int16, "idx")
    n = idx.numel()
    out = torch.empty(max(int(lib().snn_packed_index_bytes(n, tau)) // 4, 1), dtype=torch.int32, device=idx.device)
    _check(lib().snn_pack_indices(_ptr(idx), n, tau, _ptr(out), _stream()), "snn_pack_indices")
    return out


def snn_subbit_prepare_packed(desc, codebook, idx_packed, tau, alpha, workspace=None):
    _dev(codebook, torch.int16, "codebook")
    _dev(idx_packed, torch.int32, "idx_packed")
    _dev(alpha, torch.float32, "alpha")
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_SUBBIT, codebook.device)
    _check(lib().snn_subbit_prepare_packed(ctypes.byref(desc), _ptr(codebook), _ptr(idx_packed), tau, _ptr(alpha),
                                           _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_prepare_packed")
    return workspace


def snn_subbit_conv2d_prepared(desc, x, alpha, workspace, y=None):
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    _check(lib().snn_subbit_conv2d_prepared(ctypes.byref(desc), _ptr(x), _ptr(alpha), _ptr(y), _ptr(workspace),
                                            workspace.numel(), _stream()), "snn_subbit_conv2d_prepared")
    return y


def snn_subbit_forward(desc, x, w, codebook, alpha, idx_out=None, y=None, workspace=None):
    """One layer's forward pass: x float32 NCHW, w float32 [C_out][C_in][9] (or [C_out*C_in][9]),
    codebook int16 [K], alpha float32 [C_out] -> (y float32 [N][C_out][Ho][Wo], idx int16 [C_out][C_in])."""
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    _dev(codebook, torch.int16, "codebook")
    _dev(alpha, torch.float32, "alpha")
    if w.numel() != desc.C_out * desc.C_in * 9:
        raise ValueError("w has the wrong size")
    if idx_out is None:
        idx_out = torch.empty((desc.C_out, desc.C_in), dtype=torch.int16, device=x.device)
    _dev(idx_out, torch.int16, "idx_out")
    if idx_out.numel() != desc.C_out * desc.C_in:
        raise ValueError("idx_out has the wrong size")
    y = _conv_out(desc, y, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_FORWARD, x.device)
    _check(lib().snn_subbit_forward(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(codebook), _ptr(alpha), _ptr(idx_out),
                                    _ptr(y), _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_forward")
    return y, idx_out


def _sign_out(desc, out, device):
    Ho, Wo = out_hw(desc)
    words = desc.N * desc.C_out * Ho * ((Wo + 31) // 32)
    if out is None:
        out = torch.empty(words, dtype=torch.int32, device=device)
    _dev(out, torch.int32, "out")
    if out.numel() < words:
        raise ValueError("packed output too small")
    return out


def snn_subbit_conv2d_sign(desc, x, codebook, idx, alpha, beta, out=None, workspace=None):
    """x: packed int32 rows; -> packed int32 rows [N][C_out][Ho][ceil(Wo/32)] of (S*alpha + beta >= 0)."""
    _dev(x, torch.int32, "x")
    _dev(codebook, torch.int16, "codebook")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    _dev(beta, torch.float32, "beta")
    out = _sign_out(desc, out, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_SUBBIT, x.device)
    _check(lib().snn_subbit_conv2d_sign(ctypes.byref(desc), _ptr(x), _ptr(codebook), _ptr(idx), _ptr(alpha), _ptr(beta),
                                        _ptr(out), _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_conv2d_sign")
    return out


def snn_subbit_prepare_sign(desc, codebook, idx, alpha, beta, workspace=None):
    _dev(codebook, torch.int16, "codebook")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    _dev(beta, torch.float32, "beta")
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_SUBBIT, codebook.device)
    _check(lib().snn_subbit_prepare_sign(ctypes.byref(desc), _ptr(codebook), _ptr(idx), _ptr(alpha), _ptr(beta),
                                         _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_prepare_sign")
    return workspace


def snn_subbit_conv2d_sign_prepared(desc, x, workspace, out=None):
    _dev(x, torch.int32, "x")
    out = _sign_out(desc, out, x.device)
    _check(lib().snn_subbit_conv2d_sign_prepared(ctypes.byref(desc), _ptr(x), _ptr(out), _ptr(workspace),
                                                 workspace.numel(), _stream()), "snn_subbit_conv2d_sign_prepared")
    return out


def layer_weights_array(layers):
    """layers: list of dicts with keys desc, w, codebook, alpha, idx_out, workspace and optionally beta
    (torch tensors) -> a ctypes array for snn_subbit_project_prepare_many; build it once and reuse it
    (the tensors must stay alive)."""
    arr = (snn_layer_weights * len(layers))()
    for i, L in enumerate(layers):
        _dev(L["w"], torch.float32, "w")
        _dev(L["codebook"], torch.int16, "codebook")
        _dev(L["alpha"], torch.float32, "alpha")
        _dev(L["idx_out"], torch.int16, "idx_out")
        d = L["desc"]
        if L["w"].numel() != d.C_out * d.C_in * 9 or L["idx_out"].numel() != d.C_out * d.C_in:
            raise ValueError("w / idx_out have the wrong size")
        arr[i].desc = d
        arr[i].w = L["w"].data_ptr()
        arr[i].codebook = L["codebook"].data_ptr()
        arr[i].alpha = L["alpha"].data_ptr()
        beta = L.get("beta")
        if beta is not None:
            _dev(beta, torch.float32, "beta")
        arr[i].beta = beta.data_ptr() if beta is not None else None
        arr[i].idx_out = L["idx_out"].data_ptr()
        arr[i].workspace = L["workspace"].data_ptr()
        arr[i].ws_bytes = L["workspace"].numel()
    return arr


def snn_subbit_project_prepare_many(arr):
    _check(lib().snn_subbit_project_prepare_many(arr, len(arr), _stream()), "snn_subbit_project_prepare_many")


def layer_io_array(layers):
    """layers: list of dicts with keys desc, x (packed int32 rows), y (float32 output), workspace (prepared) ->
    a ctypes array for snn_subbit_conv2d_prepared_many; build it once and reuse it (the tensors must stay alive)."""
    arr = (snn_layer_io * len(layers))()
    for i, L in enumerate(layers):
        _dev(L["x"], torch.int32, "x")
        _dev(L["y"], torch.float32, "y")
        d = L["desc"]
        if L["x"].numel() * 4 != snn_packed_bytes(d.N, d.C_in, d.H, d.W, SNN_ACT_BIN_ROWS):
            raise ValueError("x has the wrong size")
        if L["y"].numel() != d.N * d.C_out * ((d.H - 1) // d.stride + 1) * ((d.W - 1) // d.stride + 1):
            raise ValueError("y has the wrong size")
        arr[i].desc = d
        arr[i].x_packed = L["x"].data_ptr()
        arr[i].y_nchw = L["y"].data_ptr()
        arr[i].workspace = L["workspace"].data_ptr()
        arr[i].ws_bytes = L["workspace"].numel()
    return arr


def snn_subbit_conv2d_prepared_many(arr):
    _check(lib().snn_subbit_conv2d_prepared_many(arr, len(arr), _stream()), "snn_subbit_conv2d_prepared_many")


def layer_forward_array(layers):
    """layers: list of dicts with keys desc, x (float32 NCHW), w (float32 [C_out*C_in][9]), codebook, alpha, idx_out
    (int16 [C_out*C_in]), y (float32 output), workspace (SNN_WS_FORWARD bytes) -> a ctypes array for
    snn_subbit_forward_many; build it once and reuse it (the tensors must stay alive)."""
    arr = (snn_layer_forward * len(layers))()
    for i, L in enumerate(layers):
        d = L["desc"]
        _dev(L["x"], torch.float32, "x")
        _dev(L["w"], torch.float32, "w")
        _dev(L["codebook"], torch.int16, "codebook")
        _dev(L["alpha"], torch.float32, "alpha")
        _dev(L["idx_out"], torch.int16, "idx_out")
        _dev(L["y"], torch.float32, "y")
        if L["x"].numel() != d.N * d.C_in * d.H * d.W or L["w"].numel() != d.C_out * d.C_in * 9:
            raise ValueError("x or w has the wrong size")
        if L["codebook"].numel() != d.K or L["alpha"].numel() != d.C_out or L["idx_out"].numel() != d.C_out * d.C_in:
            raise ValueError("codebook, alpha or idx_out has the wrong size")
        if L["y"].numel() != d.N * d.C_out * ((d.H - 1) // d.stride + 1) * ((d.W - 1) // d.stride + 1):
            raise ValueError("y has the wrong size")
        arr[i].desc = d
        arr[i].x_nchw = L["x"].data_ptr()
        arr[i].w = L["w"].data_ptr()
        arr[i].codebook = L["codebook"].data_ptr()
        arr[i].alpha = L["alpha"].data_ptr()
        arr[i].idx_out = L["idx_out"].data_ptr()
        arr[i].y_nchw = L["y"].data_ptr()
        arr[i].workspace = L["workspace"].data_ptr()
        arr[i].ws_bytes = L["workspace"].numel()
    return arr


def snn_subbit_forward_many(arr):
    _check(lib().snn_subbit_forward_many(arr, len(arr), _stream()), "snn_subbit_forward_many")


def snn_subbit_forward_sign(desc, x, w, codebook, alpha, beta, idx_out=None, out=None, workspace=None):
    """x: packed int32 rows, w float32 [C_out*C_in][9] -> (packed int32 rows of the output signs, idx int16)."""
    _dev(x, torch.int32, "x")
    _dev(w, torch.float32, "w")
    _dev(codebook, torch.int16, "codebook")
    _dev(alpha, torch.float32, "alpha")
    _dev(beta, torch.float32, "beta")
    if w.numel() != desc.C_out * desc.C_in * 9:
        raise ValueError("w has the wrong size")
    if idx_out is None:
        idx_out = torch.empty((desc.C_out, desc.C_in), dtype=torch.int16, device=x.device)
    _dev(idx_out, torch.int16, "idx_out")
    out = _sign_out(desc, out, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_SUBBIT, x.device)
    _check(lib().snn_subbit_forward_sign(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(codebook), _ptr(alpha), _ptr(beta),
                                         _ptr(idx_out), _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
           "snn_subbit_forward_sign")
    return out, idx_out


def snn_project_backward(w, g_wbar, idx, K, g_w=None, g_p=None, workspace=None):
    """w, g_wbar float32 [n][9], idx int16 [n] -> (g_w float32 [n][9], g_p float32 [K][9])."""
    _dev(w, torch.float32, "w")
    _dev(g_wbar, torch.float32, "g_wbar")
    _dev(idx, torch.int16, "idx")
    n = w.numel() // 9
    if g_wbar.numel() != n * 9 or idx.numel() != n:
        raise ValueError("w, g_wbar and idx disagree on the number of kernels")
    if g_w is None:
        g_w = torch.empty((n, 9), dtype=torch.float32, device=w.device)
    if g_p is None:
        g_p = torch.empty((K, 9), dtype=torch.float32, device=w.device)
    _dev(g_w, torch.float32, "g_w")
    _dev(g_p, torch.float32, "g_p")
    if workspace is None:
        workspace = torch.empty(max(int(lib().snn_project_backward_workspace_bytes(n, K)), 256), dtype=torch.uint8, device=w.device)
    _check(lib().snn_project_backward(_ptr(w), _ptr(g_wbar), _ptr(idx), n, K, _ptr(g_w), _ptr(g_p), _ptr(workspace),
                                      workspace.numel(), _stream()), "snn_project_backward")
    return g_w, g_p


def snn_subset_update(p, m, theta):
    """p float32 [K][9], m int8 [K][9] (updated in place) -> (codebook int16 [K], dup uint8 [K])."""
    _dev(p, torch.float32, "p")
    _dev(m, torch.int8, "m")
    K = p.numel() // 9
    if m.numel() != K * 9:
        raise ValueError("p and m disagree on K")
    cb = torch.empty(K, dtype=torch.int16, device=p.device)
    dup = torch.empty(K, dtype=torch.uint8, device=p.device)
    _check(lib().snn_subset_update(_ptr(p), _ptr(m), float(theta), K, _ptr(cb), _ptr(dup), _stream()), "snn_subset_update")
    return cb, dup


def snn_subbit_conv1x1(desc, x, codebook8, idx, alpha, y=None, workspace=None):
    """x: packed int32 channels layout; codebook8 int16 [K] (8-bit codes); idx int16 [C_out][C_in/8]."""
    _dev(x, torch.int32, "x")
    _dev(codebook8, torch.int16, "codebook8")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_CONV1X1, x.device)
    _check(lib().snn_subbit_conv1x1(ctypes.byref(desc), _ptr(x), _ptr(codebook8), _ptr(idx), _ptr(alpha), _ptr(y),
                                    _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_conv1x1")
    return y


def snn_subbit_conv1x1_prepare(desc, codebook8, idx, alpha, workspace=None):
    """Tables of a 1x1 layer -> `workspace` (returned); then any number of snn_subbit_conv1x1_prepared calls."""
    _dev(codebook8, torch.int16, "codebook8")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_CONV1X1, idx.device)
    _check(lib().snn_subbit_conv1x1_prepare(ctypes.byref(desc), _ptr(codebook8), _ptr(idx), _ptr(alpha), _ptr(workspace),
                                            workspace.numel(), _stream()), "snn_subbit_conv1x1_prepare")
    return workspace


def snn_subbit_conv1x1_prepared(desc, x, workspace, y=None):
    _dev(x, torch.int32, "x")
    y = _conv_out(desc, y, x.device)
    _check(lib().snn_subbit_conv1x1_prepared(ctypes.byref(desc), _ptr(x), _ptr(y), _ptr(workspace), workspace.numel(), _stream()),
           "snn_subbit_conv1x1_prepared")
    return y


def snn_bnn_conv2d(desc, x, w9, alpha, y=None, workspace=None):
    """x: packed int32 (channels layout) or float32 NCHW per desc.act; w9 int16 [C_out][C_in]."""
    _dev(w9, torch.int16, "w9")
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_BNN, x.device)
    _check(lib().snn_bnn_conv2d(ctypes.byref(desc), _ptr(x), _ptr(w9), _ptr(alpha), _ptr(y), _ptr(workspace),
                                workspace.numel(), _stream()), "snn_bnn_conv2d")
    return y


def snn_bnn_prepare(desc, w9, workspace):
    """The weights-side half of snn_bnn_conv2d: w9 -> bit planes and border corrections in `workspace`."""
    _dev(w9, torch.int16, "w9")
    _check(lib().snn_bnn_prepare(ctypes.byref(desc), _ptr(w9), _ptr(workspace), workspace.numel(), _stream()),
           "snn_bnn_prepare")


def snn_bnn_conv2d_prepared(desc, x, alpha, workspace, y=None):
    """The convolution half of snn_bnn_conv2d, from a workspace snn_bnn_prepare has filled."""
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    _check(lib().snn_bnn_conv2d_prepared(ctypes.byref(desc), _ptr(x), _ptr(alpha), _ptr(y), _ptr(workspace),
                                         workspace.numel(), _stream()), "snn_bnn_conv2d_prepared")
    return y


def snn_bnn_conv2d_dense(desc, x, w9, alpha, y=None, workspace=None):
    """x: packed int32 (channels layout); w9 int16 [C_out][C_in]; the 1-bit layer on the matrix cores."""
    _dev(w9, torch.int16, "w9")
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_BNN_DENSE, x.device)
    _check(lib().snn_bnn_conv2d_dense(ctypes.byref(desc), _ptr(x), _ptr(w9), _ptr(alpha), _ptr(y), _ptr(workspace),
                                      workspace.numel(), _stream()), "snn_bnn_conv2d_dense")
    return y


def snn_subbit_conv2d_dense(desc, x, codebook, idx, alpha, y=None, workspace=None):
    """A sub-bit layer (codebook int16 [K], idx int16 [C_out][C_in]) through the dense contraction."""
    _dev(codebook, torch.int16, "codebook")
    _dev(idx, torch.int16, "idx")
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    if workspace is None:
        workspace = alloc_workspace(desc, SNN_WS_BNN_DENSE, x.device)
    _check(lib().snn_subbit_conv2d_dense(ctypes.byref(desc), _ptr(x), _ptr(codebook), _ptr(idx), _ptr(alpha), _ptr(y),
                                         _ptr(workspace), workspace.numel(), _stream()), "snn_subbit_conv2d_dense")
    return y


def snn_dense_prepare(desc, codebook, codes, workspace):
    """codebook None: codes are 9-bit kernel codes; else indices into codebook.  Fills the workspace."""
    _dev(codes, torch.int16, "codes")
    if codebook is not None:
        _dev(codebook, torch.int16, "codebook")
    _check(lib().snn_dense_prepare(ctypes.byref(desc), _ptr(codebook) if codebook is not None else None, _ptr(codes),
                                   _ptr(workspace), workspace.numel(), _stream()), "snn_dense_prepare")


def snn_dense_conv2d_prepared(desc, x, alpha, workspace, y=None):
    _dev(alpha, torch.float32, "alpha")
    y = _conv_out(desc, y, x.device)
    _check(lib().snn_dense_conv2d_prepared(ctypes.byref(desc), _ptr(x), _ptr(alpha), _ptr(y), _ptr(workspace),
                                           workspace.numel(), _stream()), "snn_dense_conv2d_prepared")
    return y


def snn_dense_conv2d_sign_prepared(desc, x, alpha, beta, workspace, out=None):
    """Packed channels in, the next layer's packed channels out (int32 [N*Ho*Wo*ceil(C_out/32)])."""
    _dev(alpha, torch.float32, "alpha")
    _dev(beta, torch.float32, "beta")
    Ho = (desc.H - 1) // desc.stride + 1
    Wo = (desc.W - 1) // desc.stride + 1
    words = snn_packed_bytes(desc.N, desc.C_out, Ho, Wo, SNN_ACT_BIN_CHANNELS) // 4
    if out is None:
        out = torch.empty(words, dtype=torch.int32, device=x.device)
    _dev(out, torch.int32, "out")
    if out.numel() < words:
        raise ValueError("out is too small")
    _check(lib().snn_dense_conv2d_sign_prepared(ctypes.byref(desc), _ptr(x), _ptr(alpha), _ptr(beta), _ptr(out),
                                                _ptr(workspace), workspace.numel(), _stream()),
           "snn_dense_conv2d_sign_prepared")
    return out


def snn_project_vectors8(w, codebook8, out=None):
    """w float32 [n][8] (or any shape with 8 n elements), codebook8 int16 [K <= 256] -> int16 [n] indices."""
    _dev(w, torch.float32, "w")
    _dev(codebook8, torch.int16, "codebook8")
    if w.numel() % 8:
        raise ValueError("w must hold whole vectors of 8")
    n = w.numel() // 8
    if out is None:
        out = torch.empty(n, dtype=torch.int16, device=w.device)
    _dev(out, torch.int16, "out")
    if out.numel() < n:
        raise ValueError("out is too small")
    _check(lib().snn_project_vectors8(_ptr(w), n, _ptr(codebook8), int(codebook8.numel()), _ptr(out), _stream()),
           "snn_project_vectors8")
    return out
