"""snn_subbit_conv2d_prepared_many (the convolutions of several prepared layers in as few launches as
possible) against the oracle, element by element and bit for bit, through every tile form of the
resident-worker kernel and through the layers it hands to the per-layer kernel; guard bytes around
every output and workspace."""
import sys

import numpy as np
import pytest
import torch

from paper_2110_09195_amd import binding as B
from paper_2110_09195_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, file=sys.stderr, flush=True)


def _make(oracle, seed, N, C_in, C_out, H, W, stride, K):
    g = np.random.default_rng(1000 + seed)
    x = g.standard_normal((N, C_in, H, W), dtype=np.float32)
    cb = synth.codebook(g, K)
    idx = synth.indices(g, C_out, C_in, K)
    alpha = synth.alpha(g, C_out)
    d = B.make_desc(N, C_in, C_out, H, W, stride, K, B.SNN_ACT_BIN_ROWS)
    Ho, Wo = B.out_hw(d)
    gw = G.guarded_workspace(d, B.SNN_WS_SUBBIT)
    B.snn_subbit_prepare(d, G.dev(cb), G.dev(idx), G.dev(alpha), workspace=gw.t)
    gy = G.Guarded(N * C_out * Ho * Wo, torch.float32, fill=float("nan"))
    _, Y = oracle.conv_bin(oracle.sign(x), oracle.expand(cb, idx), alpha, stride)
    return {"desc": d, "x": B.snn_pack_activations(G.dev(x), B.SNN_ACT_BIN_ROWS), "y": gy.t.view(N, C_out, Ho, Wo),
            "workspace": gw.t, "gy": gy, "gw": gw, "Y": Y, "shape": (N, C_in, C_out, H, W, stride, K)}


def _check(layers, what):
    for L in layers:
        L["gy"].check("y of %s" % (L["shape"],))
        L["gw"].check("the workspace of %s" % (L["shape"],))
        y = L["y"].cpu().numpy()
        assert (y == L["Y"]).all(), "%s: layer %s differs from the oracle at %s" % (what, L["shape"], np.argwhere(y != L["Y"])[:5])


# N, C_in, C_out, H, W, stride, K -- one layer (at least) per tile form of the resident-worker kernel
FORMS = [
    (3, 128, 128, 7, 7, 1, 32),      # 2 x 4 blocks, one-word rows; 49-pixel planes: 4-byte stores
    (2, 30, 130, 9, 9, 1, 32),       # the same with padded channel blocks and an even C_in / odd planes
    (2, 33, 256, 12, 12, 2, 32),     # odd C_in, stride 2, planes of 36 pixels: 16-byte stores
    (2, 24, 70, 56, 56, 1, 32),      # 2 x 4 blocks, two-word rows
    (2, 24, 96, 56, 56, 2, 17),      # the same at stride 2, K not a power of two
    (1, 10, 70, 5, 70, 1, 32),       # 2 x 4 blocks, rows of three words
    (2, 64, 64, 14, 14, 1, 32),      # 4 x 2 blocks, one-word rows staged through LDS
    (2, 24, 40, 56, 56, 1, 32),      # 4 x 2 blocks, two-word rows staged through LDS
    (5, 7, 20, 40, 2, 1, 32),        # 4 x 2 blocks, rows too many to stage: loaded directly
    (2, 64, 24, 8, 8, 2, 64),        # 64 members: one input channel per matrix instruction (per-layer kernel)
    (1, 6, 10, 4, 70, 1, 32),        # 4 x 2 blocks with wide rows (per-layer kernel)
    (1, 2, 1, 1, 1, 1, 1),           # everything degenerate
]


@pytest.mark.parametrize("stack", [None, 0])
def test_many_every_form_in_one_call(oracle, stack, tune):
    """stack = 0: the launch with one workgroup per group of tiles instead of resident workers."""
    if stack is not None:
        tune("STACK", stack)
    layers = [_make(oracle, i, *c) for i, c in enumerate(FORMS)]
    io = B.layer_io_array(layers)
    for rep in range(3):             # the work counter is left at zero by every launch
        for L in layers:
            L["y"].fill_(float("nan"))
        _say("many: %d layers, call %d" % (len(layers), rep))
        B.snn_subbit_conv2d_prepared_many(io)
        _check(layers, "call %d" % rep)


@pytest.mark.parametrize("case", FORMS)
def test_many_single_layer(oracle, case):
    _say("many, one layer", case)
    layers = [_make(oracle, 50, *case)]
    B.snn_subbit_conv2d_prepared_many(B.layer_io_array(layers))
    _check(layers, "single layer")


@pytest.mark.parametrize("stack", [None, 0])
def test_many_more_layers_than_one_launch_holds(oracle, stack, tune):
    if stack is not None:
        tune("STACK", stack)
    cases = [(1, 4 + 2 * i, 8 + 8 * (i % 5), 5 + i % 3, 6 + i % 4, 1 + i % 2, 32) for i in range(19)]
    layers = [_make(oracle, 100 + i, *c) for i, c in enumerate(cases)]
    _say("many: 19 layers")
    B.snn_subbit_conv2d_prepared_many(B.layer_io_array(layers))
    _check(layers, "19 layers")


def test_many_equals_per_layer_calls_on_a_multi_tile_stack(oracle):
    """Layers big enough that every worker draws several items, some of them from different layers."""
    cases = [(16, 64, 64, 56, 56, 1, 32), (16, 64, 128, 56, 56, 2, 32), (16, 128, 128, 28, 28, 1, 32), (16, 256, 256, 14, 14, 1, 32),
             (16, 512, 512, 7, 7, 1, 32)]
    layers = []
    for i, (N, C_in, C_out, H, W, stride, K) in enumerate(cases):
        g = np.random.default_rng(2000 + i)
        x = g.standard_normal((N, C_in, H, W), dtype=np.float32)
        cb, idx, alpha = synth.codebook(g, K), synth.indices(g, C_out, C_in, K), synth.alpha(g, C_out)
        d = B.make_desc(N, C_in, C_out, H, W, stride, K, B.SNN_ACT_BIN_ROWS)
        Ho, Wo = B.out_hw(d)
        gw = G.guarded_workspace(d, B.SNN_WS_SUBBIT)
        B.snn_subbit_prepare(d, G.dev(cb), G.dev(idx), G.dev(alpha), workspace=gw.t)
        xp = B.snn_pack_activations(G.dev(x), B.SNN_ACT_BIN_ROWS)
        ref = B.snn_subbit_conv2d_prepared(d, xp, G.dev(alpha), gw.t)
        gy = G.Guarded(N * C_out * Ho * Wo, torch.float32, fill=float("nan"))
        # the oracle on the first two and the last image; the per-layer kernel (itself checked against the oracle
        # everywhere else in this suite) on all of them
        sel = [0, 1, N - 1]
        _, Y = oracle.conv_bin(oracle.sign(x[sel]), oracle.expand(cb, idx), alpha, stride)
        layers.append({"desc": d, "x": xp, "y": gy.t.view(N, C_out, Ho, Wo), "workspace": gw.t, "gy": gy, "gw": gw, "ref": ref,
                       "Y": Y, "sel": sel, "shape": cases[i]})
    io = B.layer_io_array(layers)
    for rep in range(2):
        for L in layers:
            L["y"].fill_(float("nan"))
        _say("many: multi-tile stack, call", rep)
        B.snn_subbit_conv2d_prepared_many(io)
        for L in layers:
            L["gy"].check("y")
            L["gw"].check("the workspace")
            assert torch.equal(L["y"], L["ref"]), "layer %s differs from the per-layer call" % (L["shape"],)
            assert (L["y"][L["sel"]].cpu().numpy() == L["Y"]).all(), "layer %s differs from the oracle" % (L["shape"],)


def test_many_rejections():
    d = B.make_desc(2, 8, 8, 6, 6, 1, 32, B.SNN_ACT_BIN_ROWS)
    x = torch.zeros(B.snn_packed_bytes(2, 8, 6, 6, B.SNN_ACT_BIN_ROWS) // 4, dtype=torch.int32, device="cuda")
    y = torch.zeros((2, 8, 6, 6), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(d, B.SNN_WS_SUBBIT)
    arr = B.layer_io_array([{"desc": d, "x": x, "y": y, "workspace": ws}])
    arr[0].ws_bytes = 16
    with pytest.raises(B.SnnError) as e:
        B.snn_subbit_conv2d_prepared_many(arr)
    assert e.value.status == -3
    arr[0].ws_bytes = ws.numel()
    arr[0].y_nchw = None
    with pytest.raises(B.SnnError) as e:
        B.snn_subbit_conv2d_prepared_many(arr)
    assert e.value.status == -1
    assert B.lib().snn_subbit_conv2d_prepared_many(None, 0, None) == 0


def test_config5_every_image_of_every_layer(oracle):
    """The headline workload in full, as bench.py launches it (weights-side work of all layers in one launch, packing
    per layer, all convolutions in one launch), every output of every image against the oracle."""
    layers = synth.resnet18_stack(N=64, K=32)
    st = []
    for i, L in enumerate(layers):
        g = synth.rng(5, i)
        x = synth.activations(g, L.N, L.C_in, L.H, L.W)
        cb = synth.codebook(g, L.K)
        w = synth.real_kernels(g, L.C_out * L.C_in)
        alpha = synth.alpha(g, L.C_out)
        d = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_ROWS)
        st.append({"L": L, "x": x, "cb": cb, "w": w, "alpha": alpha, "desc": d, "xd": G.dev(x), "w_d": G.dev(w), "cb_d": G.dev(cb),
                   "alpha_d": G.dev(alpha), "idx": torch.empty(L.C_out * L.C_in, dtype=torch.int16, device="cuda"),
                   "workspace": B.alloc_workspace(d, B.SNN_WS_SUBBIT),
                   "y": torch.full((L.N, L.C_out, L.H_out, L.W_out), float("nan"), dtype=torch.float32, device="cuda")})
    B.snn_subbit_project_prepare_many(B.layer_weights_array(
        [{"desc": s["desc"], "w": s["w_d"], "codebook": s["cb_d"], "alpha": s["alpha_d"], "idx_out": s["idx"], "workspace": s["workspace"]}
         for s in st]))
    for s in st:
        s["xr"] = B.snn_pack_activations(s["xd"], B.SNN_ACT_BIN_ROWS)
    B.snn_subbit_conv2d_prepared_many(B.layer_io_array([{"desc": s["desc"], "x": s["xr"], "y": s["y"], "workspace": s["workspace"]} for s in st]))
    torch.cuda.synchronize()
    for s in st:
        L = s["L"]
        _say("config 5, all 64 images:", L.name)
        idx, _ = oracle.project(s["w"], s["cb"])
        assert (G.host_u16(s["idx"]) == idx).all(), "projection of " + L.name
        _, Y = oracle.conv_bin(oracle.sign(s["x"]), oracle.expand(s["cb"], idx.reshape(L.C_out, L.C_in)), s["alpha"], L.stride)
        assert (s["y"].cpu().numpy() == Y).all(), "convolution of " + L.name


# ---- snn_subbit_forward_many: projection + tables + sign/pack of all layers in one launch, all convolutions in a second ----

def _make_forward(oracle, seed, N, C_in, C_out, H, W, stride, K):
    g = np.random.default_rng(3000 + seed)
    x = g.standard_normal((N, C_in, H, W), dtype=np.float32)
    x.flat[::11] = 0.0                      # sign(0) = +1
    cb = synth.codebook(g, K)
    w = synth.real_kernels(g, C_out * C_in)
    w[::7] = 0.0                            # ties of the projection: lowest index wins
    alpha = synth.alpha(g, C_out)
    d = B.make_desc(N, C_in, C_out, H, W, stride, K, B.SNN_ACT_BIN_ROWS)
    Ho, Wo = B.out_hw(d)
    gw = G.guarded_workspace(d, B.SNN_WS_FORWARD)
    gy = G.Guarded(N * C_out * Ho * Wo, torch.float32, fill=float("nan"))
    gi = G.Guarded(C_out * C_in, torch.int16, fill=-1)
    idx, _ = oracle.project(w, cb)
    _, Y = oracle.conv_bin(oracle.sign(x), oracle.expand(cb, idx.reshape(C_out, C_in)), alpha, stride)
    return {"desc": d, "x": G.dev(x), "w": G.dev(w), "codebook": G.dev(cb), "alpha": G.dev(alpha), "idx_out": gi.t,
            "y": gy.t.view(N, C_out, Ho, Wo), "workspace": gw.t, "gy": gy, "gw": gw, "gi": gi, "Y": Y, "idx": idx,
            "shape": (N, C_in, C_out, H, W, stride, K)}


def _check_forward(layers, what):
    _check(layers, what)
    for L in layers:
        L["gi"].check("idx_out of %s" % (L["shape"],))
        assert (G.host_u16(L["idx_out"]) == L["idx"].reshape(-1)).all(), "%s: projection of %s" % (what, L["shape"])


@pytest.mark.parametrize("stack", [None, 0])
def test_forward_many_every_form(oracle, stack, tune):
    if stack is not None:
        tune("STACK", stack)
    layers = [_make_forward(oracle, i, *c) for i, c in enumerate(FORMS)]
    arr = B.layer_forward_array(layers)
    for rep in range(2):
        for L in layers:
            L["y"].fill_(float("nan"))
            L["idx_out"].fill_(-1)
        _say("forward_many: %d layers, call %d" % (len(layers), rep))
        B.snn_subbit_forward_many(arr)
        _check_forward(layers, "call %d" % rep)


def test_forward_many_more_layers_than_one_launch_holds(oracle):
    cases = [(1, 4 + 2 * i, 8 + 8 * (i % 5), 5 + i % 3, 6 + i % 4, 1 + i % 2, 32) for i in range(19)]
    layers = [_make_forward(oracle, 100 + i, *c) for i, c in enumerate(cases)]
    _say("forward_many: 19 layers")
    B.snn_subbit_forward_many(B.layer_forward_array(layers))
    _check_forward(layers, "19 layers")


def test_forward_many_equals_forward_per_layer(oracle):
    cases = [(8, 64, 64, 56, 56, 1, 32), (8, 64, 128, 56, 56, 2, 32), (8, 256, 256, 14, 14, 1, 32), (8, 512, 512, 7, 7, 1, 32)]
    layers = [_make_forward(oracle, 200 + i, *c) for i, c in enumerate(cases)]
    B.snn_subbit_forward_many(B.layer_forward_array(layers))
    _check_forward(layers, "multi-tile stack")
    for L in layers:
        d = L["desc"]
        y1, idx1 = B.snn_subbit_forward(d, L["x"], L["w"], L["codebook"], L["alpha"])
        assert torch.equal(y1.view(-1), L["y"].view(-1)) and torch.equal(idx1.view(-1), L["idx_out"].view(-1))


def test_forward_many_rejections():
    d = B.make_desc(2, 8, 8, 6, 6, 1, 32, B.SNN_ACT_BIN_ROWS)
    L = {"desc": d, "x": torch.zeros((2, 8, 6, 6), device="cuda"), "w": torch.zeros((64, 9), device="cuda"),
         "codebook": torch.arange(32, dtype=torch.int16, device="cuda"), "alpha": torch.ones(8, device="cuda"),
         "idx_out": torch.zeros(64, dtype=torch.int16, device="cuda"), "y": torch.zeros((2, 8, 6, 6), device="cuda"),
         "workspace": B.alloc_workspace(d, B.SNN_WS_FORWARD)}
    arr = B.layer_forward_array([L])
    arr[0].ws_bytes = B.snn_workspace_bytes(d, B.SNN_WS_SUBBIT)          # the convolution's share alone is too small
    with pytest.raises(B.SnnError) as e:
        B.snn_subbit_forward_many(arr)
    assert e.value.status == -3
    arr[0].ws_bytes = L["workspace"].numel()
    arr[0].w = None
    with pytest.raises(B.SnnError) as e:
        B.snn_subbit_forward_many(arr)
    assert e.value.status == -1
    arr[0].w = L["w"].data_ptr()
    arr[0].desc.K = 512
    with pytest.raises(B.SnnError) as e:
        B.snn_subbit_forward_many(arr)
    assert e.value.status == -2
    assert B.lib().snn_subbit_forward_many(None, 0, None) == 0
