"""The C-ABI library loads and exports what include/snn.h declares (CPU only: no compute call)."""
import ctypes
import os
import re

import pytest

from paper_2110_09195_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "snn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(snn_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2110_09195_amd import build
        build.build()
    return binding.lib()


def test_header_declares_the_boundary():
    names = _declared()
    for required in ("snn_pack_activations", "snn_project_kernels", "snn_subbit_conv2d", "snn_bnn_conv2d"):
        assert required in names
    assert sorted(binding.EXPORTS) == names


def test_every_declared_symbol_is_exported(L):
    for name in _declared():
        assert hasattr(L, name), name
        assert ctypes.cast(getattr(L, name), ctypes.c_void_p).value


def test_status_strings(L):
    assert binding.status_string(0) == "SNN_OK"
    assert binding.status_string(-1) == "SNN_ERR_INVALID_ARG"
    assert binding.status_string(-2) == "SNN_ERR_UNSUPPORTED"
    assert binding.status_string(-3) == "SNN_ERR_WORKSPACE"
    assert binding.status_string(-4) == "SNN_ERR_LAUNCH"
    assert binding.status_string(-99) == "SNN_ERR_UNKNOWN"


def test_packed_bytes(L):
    assert binding.snn_packed_bytes(2, 3, 4, 33, binding.SNN_ACT_BIN_ROWS) == 2 * 3 * 4 * 2 * 4
    assert binding.snn_packed_bytes(2, 40, 4, 5, binding.SNN_ACT_BIN_CHANNELS) == 2 * 4 * 5 * 2 * 4
    assert binding.snn_packed_bytes(2, 3, 4, 5, binding.SNN_ACT_F32) == 2 * 3 * 4 * 5 * 4
    assert binding.snn_packed_bytes(0, 3, 4, 5, binding.SNN_ACT_BIN_ROWS) == 0
    assert binding.snn_packed_bytes(2, 3, 4, 5, 7) == 0


def test_workspace_bytes_and_rejections(L):
    d = binding.make_desc(128, 256, 256, 14, 14, 1, 32, binding.SNN_ACT_BIN_ROWS)
    assert binding.snn_workspace_bytes(d, binding.SNN_WS_SUBBIT) > 256 * 256 * 2
    assert binding.snn_workspace_bytes(d, binding.SNN_WS_BNN) == 0        # rows layout: not for the 1-bit kernel
    d.act = binding.SNN_ACT_BIN_CHANNELS
    assert binding.snn_workspace_bytes(d, binding.SNN_WS_BNN) >= 256 * 9 * 8 * 4
    assert binding.snn_workspace_bytes(d, binding.SNN_WS_SUBBIT) == 0
    for field, bad in (("stride", 3), ("K", 0), ("K", 513), ("N", 0), ("C_in", 0), ("act", 9)):
        d = binding.make_desc(1, 32, 32, 8, 8, 1, 32, binding.SNN_ACT_BIN_ROWS)
        setattr(d, field, bad)
        assert binding.snn_workspace_bytes(d, binding.SNN_WS_SUBBIT) == 0, field
    assert binding.snn_workspace_bytes(binding.make_desc(1, 32, 32, 8, 8), 5) == 0


def test_invalid_arguments_are_status_codes_not_crashes(L):
    d = binding.make_desc(1, 32, 32, 8, 8, 1, 32, binding.SNN_ACT_BIN_ROWS)
    null = ctypes.c_void_p(0)
    assert L.snn_subbit_conv2d(ctypes.byref(d), null, null, null, null, null, null, 0, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_bnn_conv2d(ctypes.byref(d), null, null, null, null, null, 0, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_bnn_prepare(ctypes.byref(d), null, null, 0, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_bnn_conv2d_prepared(ctypes.byref(d), null, null, null, null, 0, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_subbit_forward(ctypes.byref(d), null, null, null, null, null, null, null, 0, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_pack_activations(null, null, 1, 1, 1, 1, 0, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_project_kernels(null, 4, null, 32, null, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_subbit_conv2d(None, null, null, null, null, null, null, 0, null) == binding.SNN_ERR_INVALID_ARG
    # layout / size checks happen before any device work
    one = ctypes.c_void_p(256)   # never dereferenced: the calls below are rejected first
    assert L.snn_pack_activations(one, one, 1, 1, 1, 1, binding.SNN_ACT_F32, null) == binding.SNN_ERR_INVALID_ARG
    assert L.snn_project_kernels(one, 4, one, 513, one, null) == binding.SNN_ERR_INVALID_ARG
    d.act = binding.SNN_ACT_BIN_CHANNELS
    assert L.snn_subbit_conv2d(ctypes.byref(d), one, one, one, one, one, one, 1 << 20, null) == binding.SNN_ERR_UNSUPPORTED
    d.act = binding.SNN_ACT_BIN_ROWS
    assert L.snn_bnn_conv2d(ctypes.byref(d), one, one, one, one, one, 1 << 20, null) == binding.SNN_ERR_UNSUPPORTED
    assert L.snn_subbit_conv2d(ctypes.byref(d), one, one, one, one, one, one, 16, null) == binding.SNN_ERR_WORKSPACE
    # a workspace of sufficient size at an address that is not a multiple of 256 is refused too
    odd = ctypes.c_void_p(256 + 16)
    assert L.snn_subbit_conv2d(ctypes.byref(d), one, one, one, one, one, odd, 1 << 30, null) == binding.SNN_ERR_WORKSPACE
    d.act = binding.SNN_ACT_BIN_CHANNELS
    assert L.snn_bnn_conv2d(ctypes.byref(d), one, one, one, one, odd, 1 << 30, null) == binding.SNN_ERR_WORKSPACE
    # the one-call forward pass: binary activations only, and its own workspace size
    assert L.snn_subbit_forward(ctypes.byref(d), one, one, one, one, one, one, one, 1 << 30, null) == binding.SNN_ERR_UNSUPPORTED
    d.act = binding.SNN_ACT_BIN_ROWS
    assert L.snn_subbit_forward(ctypes.byref(d), one, one, one, one, one, one, one, 16, null) == binding.SNN_ERR_WORKSPACE
    assert L.snn_subbit_forward(ctypes.byref(d), one, one, one, one, one, one, odd, 1 << 30, null) == binding.SNN_ERR_WORKSPACE
    ws_conv = binding.snn_workspace_bytes(d, binding.SNN_WS_SUBBIT)
    ws_fwd = binding.snn_workspace_bytes(d, binding.SNN_WS_FORWARD)
    assert ws_fwd >= ws_conv + binding.snn_packed_bytes(d.N, d.C_in, d.H, d.W, binding.SNN_ACT_BIN_ROWS)
    d.act = binding.SNN_ACT_F32
    assert binding.snn_workspace_bytes(d, binding.SNN_WS_FORWARD) == 0


def test_tuning_knobs_and_slots(L, tune):
    B = binding
    for knob in range(B.SNN_TUNE_COUNT):
        assert B.snn_get_tuning(knob) == B.SNN_TUNE_AUTO
    assert B.snn_get_tuning(99) == B.SNN_TUNE_AUTO
    assert L.snn_set_tuning(99, 1) == B.SNN_ERR_INVALID_ARG
    assert L.snn_set_tuning(B.SNN_TUNE_MFMA_TILE, 33) == B.SNN_ERR_INVALID_ARG
    assert L.snn_set_tuning(B.SNN_TUNE_MFMA_KS, 3) == B.SNN_ERR_INVALID_ARG
    assert L.snn_set_tuning(B.SNN_TUNE_STACK, 2) == B.SNN_ERR_INVALID_ARG
    # slots per channel of the form a layer is launched in (Sec. 4.5: the gather needs one)
    rows = B.SNN_ACT_BIN_ROWS
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 256, 256, 14, 14, 1, 32, rows)) == 32
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 256, 256, 14, 14, 1, 64, rows)) == 64
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 256, 256, 14, 14, 1, 512, rows)) == 0
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 1, 256, 14, 14, 1, 32, rows)) == 0
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 64, 64, 8, 8, 1, 32, B.SNN_ACT_F32)) == 0
    assert B.snn_subbit_slots_per_channel(B.make_desc(256, 512, 512, 7, 7, 1, 16, rows)) == 16   # long channel runs
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 64, 64, 56, 56, 1, 16, rows)) == 32
    tune("MFMA_QUAD", 0)
    assert B.snn_get_tuning(B.SNN_TUNE_MFMA_QUAD) == 0
    assert B.snn_subbit_slots_per_channel(B.make_desc(256, 512, 512, 7, 7, 1, 16, rows)) == 32
    tune("SUBBIT_MFMA", 0)
    assert B.snn_subbit_slots_per_channel(B.make_desc(64, 256, 256, 14, 14, 1, 32, rows)) == 0
    bad = B.make_desc(64, 256, 256, 14, 14, 1, 32, rows)
    bad.stride = 3
    assert L.snn_subbit_slots_per_channel(ctypes.byref(bad)) == B.SNN_ERR_INVALID_ARG


def test_workspace_covers_both_pixel_block_forms(L, tune):
    """The plain and the sign-epilogue calls cut the pixels differently and can pick different table layouts
    (four channels per step only in one of them): the reported size is the larger of the two.  Shapes on which
    the two differ, with the byte counts of the larger layout worked out by hand: selector rows of
    ceil(C_in / 4) * 4 * COP words + finishing table + table image + the stack kernel's tables."""
    B = binding
    for N, C_in in ((112, 386), (224, 258)):
        d = B.make_desc(N, C_in, 256, 14, 14, 1, 16, B.SNN_ACT_BIN_ROWS)
        COP = 256
        sel = (C_in + 3) // 4 * 4 * COP * 4
        assert B.snn_workspace_bytes(d, B.SNN_WS_SUBBIT) >= sel + COP * 16 * 8 + 512 * 48
        tune("MFMA_QUAD", 0)
        smaller = B.snn_workspace_bytes(d, B.SNN_WS_SUBBIT)
        tune("MFMA_QUAD", B.SNN_TUNE_AUTO)
        assert smaller < B.snn_workspace_bytes(d, B.SNN_WS_SUBBIT)
