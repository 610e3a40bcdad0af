#!/usr/bin/env python3
"""Benchmark of the sub-bit 3x3 convolution path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet18|cfg3|cfg4] [--no-cpu]

One "step" is one pass of the whole path over one batch of synthetic input, i.e. the forward
lines of Alg. 1 for every 3x3 layer of the workload: project the real-valued kernels onto the
layer's subset (all layers in one launch, snn_subbit_project_prepare_many), then per layer
binarise and pack the activations and run the sub-bit convolution (stage 1, stage 2, alpha
scaling).  The same work as one snn_subbit_forward call per layer and through the three
separate entry points (snn_project_kernels, snn_pack_activations, snn_subbit_conv2d) is timed
next to it.  Inputs are resident in HBM before the timed region.  The same layers are
then run through the library's 1-bit XNOR/popcount kernel (snn_bnn_conv2d on the decoded
kernels) for the speed-up.

Prints ONE JSON line (metric of the benchmark spec: GOPS-equivalent of the dense convolution the
layers equal, plus the speed-up over the 1-bit kernel), with a `roofline` object for the
dominant kernel and a `cpu_baseline` object (the CPU oracle timed on a bounded sample).
Per-layer detail goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 CUs x 4 SIMD x 16 lanes x 2.4 GHz plain 32-bit VALU operations per second
# (= the 157.3 TFLOP/s fp32 vector peak / 2 for FMA / 2 for the packed form).
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
# LDS: 128 bytes per clock per CU.
LDS_PEAK_BYTES = 256 * 128 * 2.4e9
HBM_PEAK_BYTES = 8.0e12
# Dense matrix-core peak for FP6 / FP4 operands (the sub-bit kernel's v_mfma_scale_f32_32x32x64_f8f6f4).
MFMA_FP6_FP4_PEAK_FLOPS = 10.1e15


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet18", choices=["resnet18", "cfg3", "cfg4", "cfg1"])
    ap.add_argument("--K", type=int, default=32)
    ap.add_argument("--layer", default=None, help="one custom layer instead of a workload: N,C_in,C_out,H,W,stride")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the chained 1-bit stack and the training-side timings (profiling runs: every launch of a "
                         "kernel then belongs to the headline path or to the 1-bit baseline)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB elementwise copy kernel once (reference for the HBM byte counters)")
    return ap.parse_args()


def _measured_traffic(args):
    """HBM bytes per step of the sub-bit kernels from the committed rocprofv3 --pmc passes
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy kernel; profiles/subbit_stack_resnet18_b64_hbm_traffic.txt).
    Only for the workload they were taken on; None otherwise."""
    path = os.path.join(ROOT, "profiles", "subbit_stack_resnet18_b64_hbm_traffic.txt")
    if args.layer or args.workload != "resnet18" or args.K != 32 or not os.path.exists(path):
        return None
    try:
        with open(path) as f:
            d = json.loads("".join(l for l in f if not l.startswith("#")))
        return {"bytes": d["bytes"], "fetch_bytes": d["fetch_bytes"], "write_bytes": d["write_bytes"],
                "unit": "HBM bytes per step, all 16 launches (rocprofv3 FETCH_SIZE/WRITE_SIZE, copy-kernel scaled)"}
    except (OSError, ValueError, KeyError):
        return None


def dense_ops_of(layers):
    return sum(L.dense_ops for L in layers)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over the batch without "
              "communication; see DESIGN.md); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2110_09195_amd import accounting, synth
    from paper_2110_09195_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    B.lib()

    if args.layer:
        N, Ci, Co, H, W, st_ = [int(v) for v in args.layer.split(",")]
        layers = [synth.Layer("custom", N=N, C_in=Ci, C_out=Co, H=H, W=W, stride=st_, K=args.K)]
        wname = "custom layer %s, K=%d" % (args.layer, args.K)
        cfg_no = 9
    elif args.workload == "resnet18":
        layers = synth.resnet18_stack(N=64, K=args.K)
        wname = "ResNet-18 3x3 conv stack (16 layers), batch 64, 224x224 shapes, binary activations, K=%d" % args.K
        cfg_no = 5
    elif args.workload == "cfg3":
        layers = [synth.CFG3]
        wname = "ResNet-18 stage-3 layer, batch 128, 256->256, 14x14, K=32, Zipf indices"
        cfg_no = 3
    elif args.workload == "cfg4":
        layers = [synth.cfg4(args.K)]
        wname = "ResNet-34 stage-4 layer, batch 256, 512->512, 7x7, K=%d" % args.K
        cfg_no = 4
    else:
        layers = [synth.CFG1]
        wname = "ResNet-20 stage-1 layer, batch 8, 16->16, 32x32, K=32"
        cfg_no = 1

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).cuda()

    if args.calibrate_copy:
        # 64 Mi floats read + 64 Mi floats written by one elementwise kernel: the known-size reference that
        # FETCH_SIZE / WRITE_SIZE readings of the conv kernels are scaled by (see the design doc / profiles/)
        ca = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        cb = torch.empty_like(ca)
        torch.add(ca, 1.0, out=cb)
        torch.cuda.synchronize()
        del ca, cb

    # ---- resident inputs and buffers -------------------------------------------------------------
    st = []
    for i, L in enumerate(layers):
        g = synth.rng(cfg_no, i)
        s = {"L": L}
        s["x"] = dev(synth.activations(g, L.N, L.C_in, L.H, L.W))
        s["cb"] = dev(synth.codebook(g, L.K))
        if args.workload == "cfg3":
            # Zipf-skewed indices: real-valued kernels are drawn around the subset members the
            # skewed indices name, so that projection reproduces a skewed index map
            idx0 = synth.indices(g, L.C_out, L.C_in, L.K, "zipf")
            cbh = s["cb"].cpu().numpy().view(np.uint16)
            members = np.array([[1.0 if (int(c) >> (8 - t)) & 1 else -1.0 for t in range(9)] for c in cbh], dtype=np.float32)
            w = members[idx0.reshape(-1)] + 0.3 * synth.real_kernels(g, L.C_out * L.C_in)
        else:
            w = synth.real_kernels(g, L.C_out * L.C_in)
        s["w"] = dev(w.astype(np.float32))
        s["alpha"] = dev(synth.alpha(g, L.C_out))
        s["idx"] = torch.empty(L.C_out * L.C_in, dtype=torch.int16, device="cuda")
        s["d_sub"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_ROWS)
        s["d_bnn"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, 512, B.SNN_ACT_BIN_CHANNELS)
        s["xr"] = torch.empty(B.snn_packed_bytes(L.N, L.C_in, L.H, L.W, B.SNN_ACT_BIN_ROWS) // 4, dtype=torch.int32, device="cuda")
        s["xc"] = torch.empty(B.snn_packed_bytes(L.N, L.C_in, L.H, L.W, B.SNN_ACT_BIN_CHANNELS) // 4, dtype=torch.int32, device="cuda")
        s["y"] = torch.empty((L.N, L.C_out, L.H_out, L.W_out), dtype=torch.float32, device="cuda")
        s["yb"] = torch.empty_like(s["y"])
        s["ws_sub"] = B.alloc_workspace(s["d_sub"], B.SNN_WS_SUBBIT)
        s["ws_bnn"] = B.alloc_workspace(s["d_bnn"], B.SNN_WS_BNN)
        s["ws_fwd"] = B.alloc_workspace(s["d_sub"], B.SNN_WS_FORWARD)
        s["d_dense"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_CHANNELS)
        s["ws_dense"] = B.alloc_workspace(s["d_dense"], B.SNN_WS_BNN_DENSE)
        st.append(s)
    torch.cuda.synchronize()

    def project(s):
        B.snn_project_kernels(s["w"], s["cb"], out=s["idx"])

    def pack_rows(s):
        B.snn_pack_activations(s["x"], B.SNN_ACT_BIN_ROWS, out=s["xr"])

    def pack_channels(s):
        B.snn_pack_activations(s["x"], B.SNN_ACT_BIN_CHANNELS, out=s["xc"])

    def conv_sub(s):
        L = s["L"]
        B.snn_subbit_conv2d(s["d_sub"], s["xr"], s["cb"], s["idx"].view(L.C_out, L.C_in), s["alpha"], y=s["y"],
                            workspace=s["ws_sub"])

    def conv_bnn(s):
        B.snn_bnn_conv2d(s["d_bnn"], s["xc"], s["w9"], s["alpha"], y=s["yb"], workspace=s["ws_bnn"])

    def conv_dense(s):
        L = s["L"]
        B.snn_subbit_conv2d_dense(s["d_dense"], s["xc"], s["cb"], s["idx"].view(L.C_out, L.C_in), s["alpha"], y=s["yb"],
                                  workspace=s["ws_dense"])

    def conv_dense_prepared(s):
        B.snn_dense_conv2d_prepared(s["d_dense"], s["xc"], s["alpha"], s["ws_dense"], y=s["yb"])

    def forward(s):
        L = s["L"]
        B.snn_subbit_forward(s["d_sub"], s["x"], s["w"], s["cb"], s["alpha"], idx_out=s["idx"].view(L.C_out, L.C_in),
                             y=s["y"], workspace=s["ws_fwd"])

    # One step = every layer's projection + sign/pack + convolution, back to back on one stream:
    # one snn_subbit_forward call per layer, which runs the small operations in one launch and the
    # convolution in a second.  step_separate is the same work as three calls (four launches) per
    # layer.  (Putting the small kernels on side streams, eagerly or as a captured HIP graph, was
    # measured and is slower here: the eager form is bound by the host's launch rate, the graph
    # replay runs the kernels no closer together than the single stream does.)
    def step_forward_calls():
        for s in st:
            forward(s)

    # the headline step: the weights-side work of all layers in ONE launch (projection + tables:
    # snn_subbit_project_prepare_many), then per layer sign/pack + convolution (two launches)
    prep_arr = B.layer_weights_array([{"desc": s["d_sub"], "w": s["w"], "codebook": s["cb"], "alpha": s["alpha"],
                                       "idx_out": s["idx"], "workspace": s["ws_sub"]} for s in st])

    def step():
        B.snn_subbit_project_prepare_many(prep_arr)
        for s in st:
            pack_rows(s)
            B.snn_subbit_conv2d_prepared(s["d_sub"], s["xr"], s["alpha"], s["ws_sub"], y=s["y"])

    def step_separate():
        for s in st:
            project(s)
            pack_rows(s)
            conv_sub(s)

    def step_bnn():
        for s in st:
            pack_channels(s)
            conv_bnn(s)

    # the same sub-bit layers (same subsets and indices) as dense FP4 contractions on the matrix
    # cores, without the sharing of Sec. 4.5: context for what that sharing buys on this chip
    def step_dense():
        for s in st:
            pack_channels(s)
            conv_dense(s)

    def step_dense_inference():
        for s in st:
            pack_channels(s)
            conv_dense_prepared(s)

    # decoded kernels for the 1-bit baseline (input preparation, outside every timed region)
    for s in st:
        project(s)
    torch.cuda.synchronize()
    for s in st:
        L = s["L"]
        s["w9"] = s["cb"][s["idx"].long()].view(L.C_out, L.C_in).contiguous()
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps between two synchronisations -------------------------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    for _ in range(args.warmup):
        step_forward_calls()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_forward_calls()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step_forward_calls = (t1 - t0) * 1e3 / args.steps

    for _ in range(args.warmup):
        step_separate()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_separate()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step_separate = (t1 - t0) * 1e3 / args.steps

    for _ in range(args.warmup):
        step_bnn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_bnn()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step_bnn = (t1 - t0) * 1e3 / args.steps

    ms_per_step_dense = ms_per_step_dense_inference = None
    if not args.headline_only:
        for _ in range(args.warmup):
            step_dense()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_dense()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step_dense = (t1 - t0) * 1e3 / args.steps
        for _ in range(args.warmup):
            step_dense_inference()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_dense_inference()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step_dense_inference = (t1 - t0) * 1e3 / args.steps

    # ---- the same stack as a chain of 1-bit activations (resnet18 workload only) ---------------------------
    # Layer i's convolution ends in the next layer's binarisation (snn_subbit_forward_sign): the packed
    # output of one layer is the packed input of the next, no fp32 activations are written and nothing
    # is packed in between.  Reported next to the headline, not as it: the headline's layers each take
    # their own fp32 input, as the workload is defined.
    chained = None
    chain_ok = not args.headline_only and args.workload == "resnet18" and not args.layer and all(
        a.C_out == b.C_in and a.H_out == b.H and a.W_out == b.W for a, b in zip(layers, layers[1:]))
    if chain_ok:
        for i, s in enumerate(st):
            L = s["L"]
            s["beta"] = dev((0.25 * synth.rng(cfg_no, 200 + i).standard_normal(L.C_out)).astype(np.float32))
            words = L.N * L.C_out * L.H_out * ((L.W_out + 31) // 32)
            s["out_bits"] = torch.empty(words, dtype=torch.int32, device="cuda")

        for s in st:
            s["ws_chain"] = B.alloc_workspace(s["d_sub"], B.SNN_WS_SUBBIT)
        chain_arr = B.layer_weights_array([{"desc": s["d_sub"], "w": s["w"], "codebook": s["cb"], "alpha": s["alpha"],
                                            "beta": s["beta"], "idx_out": s["idx"], "workspace": s["ws_chain"]} for s in st])

        def step_chained():
            B.snn_subbit_project_prepare_many(chain_arr)
            xin = B.snn_pack_activations(st[0]["x"], B.SNN_ACT_BIN_ROWS, out=st[0]["xr"])
            for s in st:
                B.snn_subbit_conv2d_sign_prepared(s["d_sub"], xin, s["ws_chain"], out=s["out_bits"])
                xin = s["out_bits"]

        for _ in range(args.warmup):
            step_chained()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_chained()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_chained = (t1 - t0) * 1e3 / args.steps
        # the same chain with the weights prepared once: one launch per layer
        for s in st:
            L = s["L"]
            s["ws_sign"] = B.snn_subbit_prepare_sign(s["d_sub"], s["cb"], s["idx"].view(L.C_out, L.C_in), s["alpha"], s["beta"])

        def step_chained_inference():
            xin = B.snn_pack_activations(st[0]["x"], B.SNN_ACT_BIN_ROWS, out=st[0]["xr"])
            for s in st:
                B.snn_subbit_conv2d_sign_prepared(s["d_sub"], xin, s["ws_sign"], out=s["out_bits"])
                xin = s["out_bits"]

        for _ in range(args.warmup):
            step_chained_inference()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_chained_inference()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_chained_inf = (t1 - t0) * 1e3 / args.steps
        # the same chain through the dense contraction (packed channels from layer to layer; context)
        for s in st:
            L = s["L"]
            B.snn_dense_prepare(s["d_dense"], s["cb"], s["idx"].view(L.C_out, L.C_in), s["ws_dense"])
            s["out_bits_c"] = torch.empty(B.snn_packed_bytes(L.N, L.C_out, L.H_out, L.W_out, B.SNN_ACT_BIN_CHANNELS) // 4,
                                          dtype=torch.int32, device="cuda")

        def step_chained_dense():
            xin = B.snn_pack_activations(st[0]["x"], B.SNN_ACT_BIN_CHANNELS, out=st[0]["xc"])
            for s in st:
                B.snn_dense_conv2d_sign_prepared(s["d_dense"], xin, s["alpha"], s["beta"], s["ws_dense"], out=s["out_bits_c"])
                xin = s["out_bits_c"]

        for _ in range(args.warmup):
            step_chained_dense()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_chained_dense()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_chained_dense = (t1 - t0) * 1e3 / args.steps
        chained = {"ms_per_step": ms_chained, "gops_eq": dense_ops_of(layers) / (ms_chained * 1e-3) / 1e9,
                   "ms_per_step_inference_dense_context": ms_chained_dense,
                   "ms_per_step_inference": ms_chained_inf,
                   "inference_step": "weights prepared once (snn_subbit_prepare_sign); pack the first input, then one "
                                     "snn_subbit_conv2d_sign_prepared launch per layer",
                   "step": "snn_subbit_project_prepare_many (projection + thresholds + tables of all layers), pack the first "
                           "input, then one snn_subbit_conv2d_sign_prepared per layer: 1-bit activations from layer to layer"}

    # the two kernels must agree (same decoded weights): a cheap end-to-end sanity check
    for s in st:
        assert torch.equal(s["y"], s["yb"]), "sub-bit and 1-bit kernels disagree on " + s["L"].name

    # ---- per-call device time with HIP events on the launch stream ---------------------------------------
    def event_time(fn, reps):
        """Median device milliseconds of fn(s) per layer over `reps` back-to-back repetitions."""
        out = []
        for s in st:
            e0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
            e1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
            fn(s)
            torch.cuda.synchronize()
            for r in range(reps):
                e0[r].record()
                fn(s)
                e1[r].record()
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) for a, b in zip(e0, e1))
            out.append(ts[len(ts) // 2])          # median: the first repetitions wait for the host
        return out

    # the convolution kernel alone (weights prepared once, as at inference): `reps` launches back to back
    # between one pair of events per layer, so that neither the preparation kernel nor the events'
    # own cost is in the figure the roofline uses
    def kernel_time(reps):
        out = []
        for s in st:
            B.snn_subbit_prepare(s["d_sub"], s["cb"], s["idx"].view(s["L"].C_out, s["L"].C_in), s["alpha"], workspace=s["ws_sub"])
            B.snn_subbit_conv2d_prepared(s["d_sub"], s["xr"], s["alpha"], s["ws_sub"], y=s["y"])
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                B.snn_subbit_conv2d_prepared(s["d_sub"], s["xr"], s["alpha"], s["ws_sub"], y=s["y"])
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / reps)
        return out

    reps = max(10, args.steps)
    t_kern = kernel_time(reps)

    # inference step: weights prepared beforehand, per layer sign/pack + convolution (two launches)
    def step_inference():
        for s in st:
            pack_rows(s)
            B.snn_subbit_conv2d_prepared(s["d_sub"], s["xr"], s["alpha"], s["ws_sub"], y=s["y"])

    for _ in range(args.warmup):
        step_inference()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_inference()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step_inference = (t1 - t0) * 1e3 / args.steps

    t_sub = event_time(conv_sub, reps)
    t_bnn = event_time(conv_bnn, reps)
    t_dense = event_time(conv_dense, reps)
    t_dense_k = event_time(conv_dense_prepared, reps)
    t_proj = event_time(project, reps)
    t_pr = event_time(pack_rows, reps)
    t_pc = event_time(pack_channels, reps)

    # training-side lines of Alg. 1 (not part of the step, which is the forward pass): the straight-through
    # estimator + gradient of the subset tensor, and the sign-memory update with the repeated-member check
    for i, s in enumerate(st):
        L = s["L"]
        gq = synth.rng(cfg_no, 300 + i)
        s["g_wbar"] = dev(gq.standard_normal((L.C_out * L.C_in, 9)).astype(np.float32))
        s["g_w"] = torch.empty_like(s["g_wbar"])
        s["g_p"] = torch.empty((L.K, 9), dtype=torch.float32, device="cuda")
        s["p"] = dev((0.01 * gq.standard_normal((L.K, 9))).astype(np.float32))
        s["m"] = torch.ones((L.K, 9), dtype=torch.int8, device="cuda")
        s["ws_bwd"] = torch.empty(max(int(B.lib().snn_project_backward_workspace_bytes(L.C_out * L.C_in, L.K)), 256),
                                  dtype=torch.uint8, device="cuda")

    def project_backward(s):
        B.snn_project_backward(s["w"], s["g_wbar"], s["idx"], s["L"].K, g_w=s["g_w"], g_p=s["g_p"], workspace=s["ws_bwd"])

    def subset_update(s):
        B.snn_subset_update(s["p"], s["m"], 1e-3)

    t_pb = event_time(project_backward, reps) if not args.headline_only else [0.0] * len(st)
    t_su = event_time(subset_update, reps) if not args.headline_only else [0.0] * len(st)
    bwd_bytes = sum(L.C_out * L.C_in * (36 + 36 + 2 + 36) for L in layers)

    # 1x1 layers of a bottleneck network (appendix, Table 5): shapes of ResNet-50 at batch 64, K = 32 members of {+-1}^8
    conv1x1 = None
    if not args.headline_only and args.workload == "resnet18" and not args.layer:
        conv1x1 = []
        for (ci, co, hw) in [(64, 256, 56), (256, 64, 56), (512, 128, 28), (128, 512, 28), (1024, 256, 14), (2048, 512, 7)]:
            gq = synth.rng(cfg_no, 400 + ci + co)
            d1 = B.make_desc(64, ci, co, hw, hw, 1, 32, B.SNN_ACT_BIN_CHANNELS)
            x1 = torch.randint(-2**31, 2**31 - 1, (B.snn_packed_bytes(64, ci, hw, hw, B.SNN_ACT_BIN_CHANNELS) // 4,),
                               dtype=torch.int32, device="cuda")
            cb1 = dev(gq.permutation(256)[:32].astype(np.uint16))
            idx1 = dev(gq.integers(0, 32, size=(co, ci // 8)).astype(np.uint16))
            al1 = dev(synth.alpha(gq, co))
            y1 = torch.empty((64, co, hw, hw), dtype=torch.float32, device="cuda")
            ws1 = B.alloc_workspace(d1, B.SNN_WS_CONV1X1)
            B.snn_subbit_conv1x1(d1, x1, cb1, idx1, al1, y=y1, workspace=ws1)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                B.snn_subbit_conv1x1(d1, x1, cb1, idx1, al1, y=y1, workspace=ws1)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / reps * 1e3
            ops = 2.0 * ci * co * 64 * hw * hw
            conv1x1.append({"layer": "%d->%d %dx%d" % (ci, co, hw, hw), "us": us, "gops_eq": ops / (us * 1e-6) / 1e9})

    dense_ops = sum(L.dense_ops for L in layers)
    gather_adds = sum(accounting.stage2_gather_adds(L) for L in layers)
    responses = sum(accounting.stage1_responses(L) for L in layers)
    out_bytes = sum(L.pixels * L.C_out * 4 for L in layers)
    in_bytes = sum(L.N * L.C_in * L.H * ((L.W + 31) // 32) * 4 for L in layers)
    idx_bytes = sum(L.C_in * L.C_out * 2 for L in layers)

    alg_hbm_bytes = float(out_bytes + in_bytes + idx_bytes)
    sub_s = sum(t_sub) * 1e-3
    kern_s = sum(t_kern) * 1e-3
    hbm = {"achieved": alg_hbm_bytes / kern_s / 1e9, "peak": HBM_PEAK_BYTES / 1e9, "unit": "GB/s",
           "frac": alg_hbm_bytes / kern_s / HBM_PEAK_BYTES}
    if all(L.K <= 32 and L.C_in >= 2 for L in layers):
        # Matrix-core kernel: stage 2 is a product with a one-hot matrix whose contraction runs over
        # (c_in, 32 subset slots), i.e. 2 * 32 flop per (pixel, c_out, c_in); stage 1 is the B operand
        # itself (a table row), so these are all the flops of the method in this formulation.
        alg_flops = 2.0 * 32.0 * gather_adds
        roofline = {
            "kernel": "subbit_mfma_kernel (all %d launches of a step; duration: snn_subbit_conv2d_prepared, the "
                      "convolution kernel alone, launched back to back between one pair of HIP events per layer)" % len(layers),
            "bound": "mfma",
            "achieved": alg_flops / kern_s / 1e12,
            "peak": MFMA_FP6_FP4_PEAK_FLOPS / 1e12,
            "unit": "TFLOP/s",
            "frac": alg_flops / kern_s / MFMA_FP6_FP4_PEAK_FLOPS,
            "traffic": _measured_traffic(args),
            "hbm": hbm,
            "avg_launch_ms": sum(t_kern) / len(t_kern),
        }
    else:
        # LDS-gather kernels (K > 32): stage 2 is one add per (pixel, c_out, c_in) with four pixels per
        # 32-bit lane operation; stage 1 one response per (pixel, c_in, k), four per lane operation.
        # Every gathered response is one byte read from LDS.
        alg_lane_ops = (gather_adds + responses) / 4.0
        alg_lds_bytes = float(gather_adds)
        roofline = {
            "kernel": "subbit_lut_kernel / subbit_wave_kernel (all %d launches of a step; duration is the "
                      "snn_subbit_conv2d call, which includes its small index-preparation kernel)" % len(layers),
            "bound": "alu",
            "achieved": alg_lane_ops / sub_s / 1e12,
            "peak": VALU_PEAK_LANE_OPS / 1e12,
            "unit": "T lane-op/s",
            "frac": alg_lane_ops / sub_s / VALU_PEAK_LANE_OPS,
            "traffic": _measured_traffic(args),
            "lds": {"achieved": alg_lds_bytes / sub_s / 1e12, "peak": LDS_PEAK_BYTES / 1e12, "unit": "TB/s",
                    "frac": alg_lds_bytes / sub_s / LDS_PEAK_BYTES},
            "hbm": hbm,
            "avg_launch_ms": sum(t_sub) / len(t_sub),
        }

    print("%-18s %9s %6s %5s | %9s %9s %7s | %8s %8s %8s" % ("layer", "pixels", "C", "K", "subbit us", "bnn us", "speedup",
                                                             "proj us", "packR us", "packC us"), file=sys.stderr)
    for L, a, b, c, d, e in zip(layers, t_sub, t_bnn, t_proj, t_pr, t_pc):
        print("%-18s %9d %3d>%-3d %4d | %9.1f %9.1f %7.2f | %8.1f %8.1f %8.1f" % (
            L.name, L.pixels, L.C_in, L.C_out, L.K, a * 1e3, b * 1e3, b / a, c * 1e3, d * 1e3, e * 1e3), file=sys.stderr)
    print("sum: subbit %.1f us, bnn %.1f us, project %.1f us, pack rows %.1f us, pack channels %.1f us; "
          "step %.1f us, bnn step %.1f us" % (sum(t_sub) * 1e3, sum(t_bnn) * 1e3, sum(t_proj) * 1e3, sum(t_pr) * 1e3,
                                                sum(t_pc) * 1e3, ms_per_step * 1e3, ms_per_step_bnn * 1e3), file=sys.stderr)
    print("the same sub-bit layers as dense FP4 contractions (snn_subbit_conv2d_dense), per layer, us, with / without "
          "the weight expansion kernel: " + " ".join("%.1f/%.1f" % (a * 1e3, b * 1e3) for a, b in zip(t_dense, t_dense_k)),
          file=sys.stderr)
    if ms_per_step_dense is not None:
        print("dense step (pack channels + dense conv per layer; the indices are given, no projection): %.1f us, with prepared weights %.1f us; dense conv "
              "calls alone: %.1f us, prepared %.1f us" % (ms_per_step_dense * 1e3, ms_per_step_dense_inference * 1e3,
                                                         sum(t_dense) * 1e3, sum(t_dense_k) * 1e3), file=sys.stderr)
    print("step as one snn_subbit_forward per layer: %.1f us" % (ms_per_step_forward_calls * 1e3), file=sys.stderr)
    print("step as three separate calls per layer: %.1f us" % (ms_per_step_separate * 1e3), file=sys.stderr)
    print("inference step (weights prepared once; pack + conv per layer): %.1f us; conv kernels alone: %.1f us" % (
        ms_per_step_inference * 1e3, sum(t_kern) * 1e3), file=sys.stderr)
    if chained is not None:
        print("chained 1-bit stack (prepare_many + conv_sign per layer): %.1f us; with prepared weights: %.1f us; the "
              "same through the dense contraction (prepared weights): %.1f us" % (
                  chained["ms_per_step"] * 1e3, chained["ms_per_step_inference"] * 1e3,
                  chained["ms_per_step_inference_dense_context"] * 1e3), file=sys.stderr)

    # ---- cpu_baseline: the oracle on a bounded sample of the same workload --------------------------------
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build()
        n_img = 64 if args.workload == "resnet18" else 16
        t_cpu = 0.0
        ops_cpu = 0
        for s in st:
            L = s["L"]
            x = s["x"][:n_img].cpu().numpy()
            w = s["w"].cpu().numpy()
            cb = s["cb"].cpu().numpy().view(np.uint16)
            alpha = s["alpha"].cpu().numpy()
            c0 = time.perf_counter()
            idx, _ = oracle.project(w, cb)
            xs = oracle.sign(x)
            _, Y = oracle.conv_bin(xs, oracle.expand(cb, idx.reshape(L.C_out, L.C_in)), alpha, L.stride)
            t_cpu += time.perf_counter() - c0
            ops_cpu += L.dense_ops // L.N * x.shape[0]
            assert (s["y"][:n_img].cpu().numpy() == Y).all(), "GPU result differs from the oracle on " + L.name
            # (s["yb"] was last written by the dense contraction of the same layer)
            assert (s["yb"][:n_img].cpu().numpy() == Y).all(), "dense-path result differs from the oracle on " + L.name
        if chained is not None:
            # the chain, first two images, layer by layer against the oracle (images are independent)
            xs = oracle.sign(st[0]["x"][:2].cpu().numpy())
            for s in st:
                L = s["L"]
                idx, _ = oracle.project(s["w"].cpu().numpy(), s["cb"].cpu().numpy().view(np.uint16))
                codes = oracle.expand(s["cb"].cpu().numpy().view(np.uint16), idx.reshape(L.C_out, L.C_in))
                want, xs = oracle.conv_sign(xs, codes, s["alpha"].cpu().numpy(), s["beta"].cpu().numpy(), L.stride)
                per_img = L.C_out * L.H_out * ((L.W_out + 31) // 32)
                got = s["out_bits"][:2 * per_img].cpu().numpy().view(np.uint32).reshape(want.shape)
                assert (got == want).all(), "chained GPU result differs from the oracle on " + L.name
                want_c = oracle.pack_channels(xs)
                got_c = s["out_bits_c"][:want_c.size].cpu().numpy().view(np.uint32).reshape(want_c.shape)
                assert (got_c == want_c).all(), "chained dense-path result differs from the oracle on " + L.name
            chained["checked"] = "first 2 images of every layer's packed output equal the oracle's chain"
        cpu = {"value": ops_cpu / t_cpu / 1e9, "unit": "GOPS-equivalent", "cores": oracle.threads(), "kind": "oracle",
               "sample": "same %d layers, first %d images of the batch (project + sign + direct conv), %.1f s" % (
                   len(layers), min(n_img, layers[0].N), t_cpu)}

    result = {
        "metric": "sub-bit 3x3 conv GOPS-equivalent (2*9*C_in*C_out*N*H_out*W_out per layer / step time) and "
                  "speed-up vs the 1-bit XNOR/popcount kernel",
        "value": dense_ops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GOPS-equivalent",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": wname,
                   "step": "snn_subbit_project_prepare_many (projection + tables of all layers, one launch), then per layer "
                           "snn_pack_activations + snn_subbit_conv2d_prepared"},
        "ms_per_step_forward_calls": ms_per_step_forward_calls,
        "forward_calls_step": "one snn_subbit_forward per layer (front kernel + convolution)",
        "ms_per_step_separate_calls": ms_per_step_separate,
        "ms_per_step_inference": ms_per_step_inference,
        "inference_step": "weights prepared once (snn_subbit_prepare); per layer snn_pack_activations + snn_subbit_conv2d_prepared",
        "conv_kernel_us_per_layer": [t * 1e3 for t in t_kern],
        "conv_only_gops_eq": dense_ops / sub_s / 1e9,
        "bnn_conv_only_gops_eq": dense_ops / (sum(t_bnn) * 1e-3) / 1e9,
        "speedup_vs_bnn_conv": sum(t_bnn) / sum(t_sub),
        "speedup_vs_bnn_step": ms_per_step_bnn / ms_per_step,
        "bnn_ms_per_step": ms_per_step_bnn,
        "breakdown_us": {"subbit_conv": sum(t_sub) * 1e3, "bnn_conv": sum(t_bnn) * 1e3, "project": sum(t_proj) * 1e3,
                         "pack_rows": sum(t_pr) * 1e3, "pack_channels": sum(t_pc) * 1e3},
        "training_side_us": {"project_backward": sum(t_pb) * 1e3, "subset_update": sum(t_su) * 1e3,
                             "project_backward_GBps": bwd_bytes / (sum(t_pb) * 1e-3) / 1e9 if sum(t_pb) > 0 else None,
                             "note": "per-call HIP-event times summed over the layers (each includes ~8 us of event and "
                                     "launch overhead); Alg. 1 backward lines, outside the step"},
        "chained_1bit_stack": chained,
        "dense_fp4_context": {
            "what": "the same sub-bit layers (subset + indices) through snn_subbit_conv2d_dense: kernels looked up and "
                    "expanded by a preparation kernel, then a dense FP4 contraction on the matrix cores without the "
                    "sharing of Sec. 4.5; context, not the paper's method.  ms_per_step = pack channels + the one-call dense "
                    "convolution per layer with the indices given (unlike the headline step it does not project the "
                    "real-valued kernels); ms_per_step_inference = pack channels + the prepared convolution per layer, "
                    "to be compared with the top-level ms_per_step_inference",
            "ms_per_step": ms_per_step_dense, "ms_per_step_inference": ms_per_step_dense_inference,
            "conv_us": sum(t_dense) * 1e3, "conv_prepared_us": sum(t_dense_k) * 1e3,
            "conv_us_per_layer": [v * 1e3 for v in t_dense],
            "conv_prepared_us_per_layer": [v * 1e3 for v in t_dense_k],
            "subbit_over_dense_conv": sum(t_sub) / sum(t_dense),
            "subbit_over_dense_conv_prepared": sum(t_kern) / sum(t_dense_k)},
        "conv1x1_resnet50_shapes": conv1x1,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
