#!/usr/bin/env python3
"""Benchmark of the sub-bit 3x3 convolution path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet18|cfg1|cfg3|cfg4] [--no-cpu]
                    [--headline-only] [--no-configs] [--no-traffic]

One "step" is one pass of the whole path over one batch of synthetic input, i.e. the forward lines of
Alg. 1 for every 3x3 layer of the workload:
  * project the real-valued kernels of all layers onto their subsets and build the convolution's tables
    (Eq. 2 / Eq. 5; one launch, snn_subbit_project_prepare_many),
  * binarise and pack every layer's fp32 input (one launch, snn_pack_activations_many),
  * the sub-bit convolutions of all layers (Sec. 4.5: stage 1, stage 2, alpha scaling; one launch,
    snn_subbit_conv2d_prepared_many).
Inputs are resident in HBM before the timed region.  The same layers then run through the library's 1-bit
XNOR/popcount kernel (snn_bnn_conv2d on the decoded kernels) for the speed-up.

Prints ONE JSON line: the metric (GOPS-equivalent of the dense convolutions the layers equal, plus the speed-up
over the 1-bit kernel), a `roofline` object for the convolution launch (algorithmic bytes, gather-adds and
responses of Sec. 4.5, the one-hot slots the kernel spends per gather as launched, fractions against the vendor
peaks and against peaks measured in this run by the probes of include/snn_peaks.h, HBM traffic from two
rocprofv3 counter passes this script starts before it touches the GPU), a `configs` array (the other four
workloads, each with its oracle check and a cold-cache series) and `cpu_baseline` (the CPU oracle timed on
a bounded sample).  Per-layer detail goes to stderr.
"""
import argparse
import csv
import json
import os
import shutil
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Vendor peaks of MI355X.
HBM_PEAK_BYTES = 8.0e12
MFMA_FP6_FP4_PEAK_FLOPS = 10.1e15          # dense FP6 / FP4 operands (v_mfma_f32_32x32x64_f8f6f4)
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz plain 32-bit VALU operations per second (= the 157.3 TFLOP/s fp32
# vector peak / 2 for FMA / 2 for the packed form)
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
MFMA_FLOP_32x32x64 = 2 * 32 * 32 * 64

COPY_CAL_BYTES = 256 * 1024 * 1024           # the copy probe of the counter passes reads and writes this much


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps before each timed region (the chip needs some 25 ms of this work to settle its clocks)")
    ap.add_argument("--workload", default="resnet18", choices=["resnet18", "cfg3", "cfg4", "cfg1"])
    ap.add_argument("--K", type=int, default=32)
    ap.add_argument("--layer", default=None, help="one custom layer instead of a workload: N,C_in,C_out,H,W,stride")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg and the oracle checks")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the step, the 1-bit baseline and the per-kernel timings of the workload (profiling "
                         "runs: no chained stack, dense context, training-side or 1x1 timings, no configs, no traffic)")
    ap.add_argument("--no-configs", action="store_true", help="skip the `configs` array (workloads 1-4)")
    ap.add_argument("--no-traffic", action="store_true", help="do not start the two rocprofv3 counter passes")
    ap.add_argument("--counter-child", action="store_true",
                    help="(internal) the program the counter passes profile: one copy probe of known size, then three "
                         "launches of the workload's convolutions")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------------------------------
# HBM traffic: two rocprofv3 --pmc passes over this script's --counter-child mode, started before the GPU is touched
# ---------------------------------------------------------------------------------------------------------------------

def _pmc_pass(counter, args, outdir):
    """One rocprofv3 pass; returns {kernel name: [KiB readings]} for `counter`, or raises."""
    rocprof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(rocprof):
        raise RuntimeError("rocprofv3 not found")
    if os.path.isdir(outdir):
        shutil.rmtree(outdir)
    os.makedirs(outdir)
    child = [sys.executable, os.path.join(ROOT, "bench.py"), "--counter-child", "--workload", args.workload, "--K", str(args.K)]
    if args.layer:
        child += ["--layer", args.layer]
    cmd = [rocprof, "--pmc", counter, "-d", outdir, "-o", "pass", "--output-format", "csv", "--"] + child
    env = dict(os.environ, TMPDIR="/tmp")
    r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=150)
    if r.returncode != 0:
        raise RuntimeError("rocprofv3 --pmc %s ended with status %d: %s" % (counter, r.returncode, r.stdout.decode(errors="replace")[-400:]))
    found = None
    for base, _, files in os.walk(outdir):
        for f in files:
            if f.endswith("counter_collection.csv"):
                found = os.path.join(base, f)
    if not found:
        raise RuntimeError("no counter_collection.csv under " + outdir)
    per = {}
    with open(found) as fh:
        for row in csv.DictReader(fh):
            if row["Counter_Name"] == counter:
                per.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
    return per


def measure_traffic(args):
    """HBM bytes of one convolution launch: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by what the same
    counter reads for the copy probe (COPY_CAL_BYTES read, COPY_CAL_BYTES written).  None (and the reason on stderr)
    if the passes cannot run."""
    out_root = os.path.join(ROOT, "gpurun_out", "bench_pmc")
    try:
        res = {}
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            per = _pmc_pass(counter, args, os.path.join(out_root, counter.lower()))
            cal = [v for k, vs in per.items() if "copy_kernel" in k for v in vs]
            conv = [v for k, vs in per.items() if "subbit_stack_kernel" in k or "subbit_mfma" in k for v in vs]
            if not cal or not conv:
                raise RuntimeError("kernels missing from the %s pass: %s" % (counter, sorted(per)))
            scale = COPY_CAL_BYTES / (sum(cal) / len(cal) * 1024.0)
            launches = 3
            # a workload the stack kernel does not hold runs as several launches per call: sum per call
            per_call = sum(conv) / launches
            res[counter] = {"bytes": per_call * 1024.0 * scale, "scale": scale, "dispatches": len(conv)}
        f, w = res["FETCH_SIZE"], res["WRITE_SIZE"]
        return {"bytes": f["bytes"] + w["bytes"], "fetch_bytes": f["bytes"], "write_bytes": w["bytes"],
                "fetch_scale": f["scale"], "write_scale": w["scale"],
                "unit": "HBM bytes per convolution launch (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, "
                        "each scaled by the same counter's reading for a copy kernel that reads and writes 256 MiB)"}
    except Exception as e:                                      # noqa: BLE001 - any failure means "not measured"
        print("bench.py: HBM traffic not measured: %s" % e, file=sys.stderr)
        return None


# ---------------------------------------------------------------------------------------------------------------------
# helpers (torch is imported in main: the counter passes start first)
# ---------------------------------------------------------------------------------------------------------------------

def workload_of(args, synth):
    if args.layer:
        N, Ci, Co, H, W, st_ = [int(v) for v in args.layer.split(",")]
        return ([synth.Layer("custom", N=N, C_in=Ci, C_out=Co, H=H, W=W, stride=st_, K=args.K)],
                "custom layer %s, K=%d" % (args.layer, args.K), 9)
    if args.workload == "resnet18":
        return (synth.resnet18_stack(N=64, K=args.K),
                "ResNet-18 3x3 conv stack (16 layers), batch 64, 224x224 shapes, binary activations, K=%d" % args.K, 5)
    if args.workload == "cfg3":
        return [synth.CFG3], "ResNet-18 stage-3 layer, batch 128, 256->256, 14x14, K=32, Zipf indices", 3
    if args.workload == "cfg4":
        return [synth.cfg4(args.K)], "ResNet-34 stage-4 layer, batch 256, 512->512, 7x7, K=%d" % args.K, 4
    return [synth.CFG1], "ResNet-20 stage-1 layer, batch 8, 16->16, 32x32, K=32", 1


class Bench:
    """Timing helpers bound to torch and the binding."""

    def __init__(self, torch, B, np, synth):
        self.torch, self.B, self.np, self.synth = torch, B, np, synth
        self._evict = None

    def dev(self, a):
        a = self.np.ascontiguousarray(a)
        if a.dtype == self.np.uint16:
            a = a.view(self.np.int16)
        return self.torch.from_numpy(a).cuda()

    def host_ms(self, fn, warmup, steps):
        """Exactly `steps` calls between two synchronisations, wall clock."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def event_avg_us(self, fn, reps):
        """`reps` launches back to back between one pair of events on the launch stream: microseconds per launch."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    def event_each_us(self, fn, reps, before=None):
        """One pair of events per launch, `before()` (untimed) ahead of each: sorted microseconds."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        e0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        e1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        for r in range(reps):
            if before is not None:
                before()
            e0[r].record()
            fn()
            e1[r].record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) * 1e3 for a, b in zip(e0, e1))

    def evict(self):
        """512 MB written between launches: more than L2 and the memory-side cache hold."""
        if self._evict is None:
            self._evict = self.torch.empty(512 * 1024 * 1024, dtype=self.torch.uint8, device="cuda")
        self._evict.fill_(1)

    def cold_us(self, fn, reps=7):
        ts = self.event_each_us(fn, reps, before=self.evict)
        return ts[len(ts) // 2]

    def layer_state(self, L, g, zipf_w=False, extra=()):
        """Resident tensors of one layer: fp32 input, subset, real-valued kernels, alpha, buffers, workspaces."""
        torch, B, np, synth = self.torch, self.B, self.np, self.synth
        s = {"L": L}
        s["x"] = self.dev(synth.activations(g, L.N, L.C_in, L.H, L.W))
        s["cb"] = self.dev(synth.codebook(g, L.K))
        if zipf_w:
            # Zipf-skewed indices: the real-valued kernels are drawn around the subset members that skewed indices
            # name, so that the projection reproduces a skewed index map
            idx0 = synth.indices(g, L.C_out, L.C_in, L.K, "zipf")
            cbh = s["cb"].cpu().numpy().view(np.uint16)
            members = np.array([[1.0 if (int(c) >> (8 - t)) & 1 else -1.0 for t in range(9)] for c in cbh], dtype=np.float32)
            w = members[idx0.reshape(-1)] + 0.3 * synth.real_kernels(g, L.C_out * L.C_in)
        else:
            w = synth.real_kernels(g, L.C_out * L.C_in)
        s["w"] = self.dev(w.astype(np.float32))
        s["alpha"] = self.dev(synth.alpha(g, L.C_out))
        s["idx"] = torch.empty(L.C_out * L.C_in, dtype=torch.int16, device="cuda")
        s["d_sub"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_ROWS)
        s["d_bnn"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, 512, B.SNN_ACT_BIN_CHANNELS)
        s["xr"] = torch.empty(B.snn_packed_bytes(L.N, L.C_in, L.H, L.W, B.SNN_ACT_BIN_ROWS) // 4, dtype=torch.int32, device="cuda")
        s["xc"] = torch.empty(B.snn_packed_bytes(L.N, L.C_in, L.H, L.W, B.SNN_ACT_BIN_CHANNELS) // 4, dtype=torch.int32, device="cuda")
        s["y"] = torch.empty((L.N, L.C_out, L.H_out, L.W_out), dtype=torch.float32, device="cuda")
        s["yb"] = torch.empty_like(s["y"])
        s["ws_sub"] = B.alloc_workspace(s["d_sub"], B.SNN_WS_SUBBIT)
        s["ws_bnn"] = B.alloc_workspace(s["d_bnn"], B.SNN_WS_BNN)
        if "forward" in extra:
            s["ws_fwd"] = B.alloc_workspace(s["d_sub"], B.SNN_WS_FORWARD)
        if "dense" in extra:
            s["d_dense"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_CHANNELS)
            s["ws_dense"] = B.alloc_workspace(s["d_dense"], B.SNN_WS_BNN_DENSE)
        return s


def measured_peaks(torch, np):
    """The yardsticks of the roofline, from the probes of include/snn_peaks.h (median of 5 measurements each; a
    measurement is four launches back to back between one pair of events, so that the 10-20 us around a single
    launch do not count against a probe of 50-200 us)."""
    from paper_2110_09195_amd import peaks as P

    def timed(fn, reps=5, inner=4):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(inner):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3 / inner)
        return sorted(ts)[len(ts) // 2]

    out = {}
    a = torch.zeros(COPY_CAL_BYTES // 4, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    out["hbm_copy_GBps"] = 2 * COPY_CAL_BYTES / timed(lambda: P.copy(b, a)) / 1e9
    big = torch.ones(1024 * 1024 * 1024 // 4, dtype=torch.int32, device="cuda")      # 1 GiB: larger than the memory-side cache
    ro = torch.empty(P.READ_BLOCKS * 256, dtype=torch.int32, device="cuda")
    out["hbm_read_GBps"] = big.numel() * 4 / timed(lambda: P.read(big, 1, ro), 3) / 1e9
    del big, ro
    out["hbm_write_GBps"] = COPY_CAL_BYTES / timed(lambda: P.fill(b, 0)) / 1e9
    out["hbm_write_nontemporal_GBps"] = COPY_CAL_BYTES / timed(lambda: P.fill(b, 1)) / 1e9
    del a, b
    o = torch.empty(2048 * 320, dtype=torch.float32, device="cuda")
    ops = [0]

    def valu():
        ops[0] = P.valu_xor_bcnt(o, 2000, 2048)
    t = timed(valu)
    out["valu_xor_bcnt_T_lane_ops"] = ops[0] / t / 1e12
    names = {0: "random", 1: "onehot_x_counts", 2: "zeros"}
    blocks, iters = 512, 4000
    for pattern in (0, 1, 2):
        n = [0]

        def mf():
            n[0] = P.mfma_f4f6(o, 0, pattern, iters, blocks)
        t = timed(mf, 3)
        clk = o[blocks * 256: blocks * 256 + blocks * 4].view(torch.int64).cpu().numpy().reshape(blocks, 2)
        mhz = clk[:, 0] / (clk[:, 1] / 100e6) / 1e6
        out["mfma_f4f6_%s_TFLOPs" % names[pattern]] = n[0] * MFMA_FLOP_32x32x64 / t / 1e12
        out["mfma_f4f6_%s_shader_MHz" % names[pattern]] = float(np.median(mhz))
        out["mfma_f4f6_%s_shader_clk_per_instr" % names[pattern]] = float(np.median(clk[:, 0]) / (iters * 8.0))
    # candidate form of stage 2 without the matrix cores (byte-SWAR adds under wave-uniform register indices)
    n_ci = 28 * 64
    rng = np.random.default_rng(1)
    idx_h = np.zeros(n_ci * 64 + 48, dtype=np.uint32)
    idx_h[:n_ci * 64] = rng.integers(0, 32, n_ci * 64)
    idx = torch.from_numpy(idx_h.view(np.int32)).cuda()
    so = torch.zeros(2048 * 256, dtype=torch.int32, device="cuda")
    g = [0]

    def swar():
        g[0] = P.swar_gather(so, idx, n_ci, 2048)
    t = timed(swar, 3)
    want = int(4 * np.array([(7 * k + 3) % 10 for k in range(32)])[idx_h[:n_ci * 64]].sum())
    out["swar_gather_T_gather_adds"] = g[0] / t / 1e12
    out["swar_gather_result_ok"] = bool((so.cpu().numpy() == want).all())
    out["onehot_mfma_T_gather_adds_at_32_slots"] = out["mfma_f4f6_onehot_x_counts_TFLOPs"] / 64.0
    out["note"] = ("probes of include/snn_peaks.h, median of 3-5 launches in this run; mfma: 512 workgroups x 4 waves x 8 "
                   "independent accumulator sets, three operand patterns (the matrix cores' clock depends on the data)")
    return out


def conv_roofline(layers, slots, t_s, peaks, accounting):
    """The roofline object of a sub-bit convolution launch (or of the launches of a list of layers): Sec. 4.5's own
    units, the unit the kernel spends per gather as launched, fractions against vendor and measured peaks."""
    gather_adds = sum(accounting.stage2_gather_adds(L) for L in layers)
    responses = sum(accounting.stage1_responses(L) for L in layers)
    out_bytes = sum(L.pixels * L.C_out * 4 for L in layers)
    in_bytes = sum(L.N * L.C_in * L.H * ((L.W + 31) // 32) * 4 for L in layers)
    idx_bytes = sum(L.C_in * L.C_out * 2 for L in layers)
    alg_bytes = float(out_bytes + in_bytes + idx_bytes)
    # flops the matrix cores execute for stage 2 as launched: 2 * slots per (pixel, c_out, c_in), channel counts
    # rounded up to what one instruction holds (2 channels at 32 slots, 4 at 16, 1 at 64)
    flops = 0.0
    for L, sl in zip(layers, slots):
        per_instr = 64 // sl
        ci = (L.C_in + per_instr - 1) // per_instr * per_instr
        flops += 2.0 * sl * L.pixels * L.C_out * ci
    t_hbm = alg_bytes / HBM_PEAK_BYTES
    t_unit = flops / MFMA_FP6_FP4_PEAK_FLOPS
    r = {
        "bound": "mfma" if t_unit >= t_hbm else "hbm",
        "alg_bytes": alg_bytes, "alg_bytes_split": {"in_packed": in_bytes, "out_f32": out_bytes, "idx_u16": idx_bytes},
        "gather_adds": gather_adds, "responses": responses,
        "unit_used": "contraction slots of v_mfma_f32_32x32x64_f8f6f4 (FP4 one-hot selector x FP6 match counts, fp32 "
                     "accumulators): stage 1 is a table row per window (no arithmetic), stage 2 spends `slots_per_channel` "
                     "multiply-adds per gather-add, of which one is not a multiplication by zero",
        "slots_per_channel": sorted(set(slots)) if len(set(slots)) > 1 else slots[0],
        "unit_flops_as_launched": flops,
        "t_kernel_us": t_s * 1e6,
        "t_floor_hbm_us": t_hbm * 1e6, "t_floor_unit_us": t_unit * 1e6,
        "achieved": (flops / t_s / 1e12) if t_unit >= t_hbm else (alg_bytes / t_s / 1e9),
        "peak": (MFMA_FP6_FP4_PEAK_FLOPS / 1e12) if t_unit >= t_hbm else (HBM_PEAK_BYTES / 1e9),
        "unit": "TFLOP/s" if t_unit >= t_hbm else "GB/s",
        "frac": max(t_hbm, t_unit) / t_s,
        "frac_hbm": t_hbm / t_s, "frac_unit": t_unit / t_s,
        "useful_frac": 2.0 * gather_adds / MFMA_FP6_FP4_PEAK_FLOPS / t_s,
        "useful_note": "one multiply-add per gather-add (Sec. 4.5) against the same peak",
    }
    if peaks:
        bw = peaks["hbm_write_nontemporal_GBps"] * 1e9        # the launch writes 96 % of its bytes, with non-temporal stores
        mf = peaks["mfma_f4f6_onehot_x_counts_TFLOPs"] * 1e12
        r["frac_vs_measured_peaks"] = max(alg_bytes / bw, flops / mf) / t_s
        r["frac_vs_measured_note"] = ("max(alg_bytes / hbm_write_nontemporal, unit_flops_as_launched / mfma_f4f6_onehot_x_counts) "
                                      "/ t_kernel, both from peaks_measured")
    return r


# ---------------------------------------------------------------------------------------------------------------------

def counter_child(args):
    """What the counter passes profile: the copy probe once, then three launches of the workload's convolutions."""
    import numpy as np
    import torch

    from paper_2110_09195_amd import binding as B
    from paper_2110_09195_amd import peaks as P
    from paper_2110_09195_amd import synth
    torch.cuda.set_device(0)
    layers, _, cfg_no = workload_of(args, synth)
    a = torch.zeros(COPY_CAL_BYTES // 4, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    io = []
    for i, L in enumerate(layers):
        g = synth.rng(cfg_no, i)
        x = torch.from_numpy(synth.activations(g, L.N, L.C_in, L.H, L.W)).cuda()
        cb = torch.from_numpy(synth.codebook(g, L.K).view(np.int16)).cuda()
        idx = torch.from_numpy(synth.indices(g, L.C_out, L.C_in, L.K).view(np.int16)).cuda()
        alpha = torch.from_numpy(synth.alpha(g, L.C_out)).cuda()
        d = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_ROWS)
        xr = B.snn_pack_activations(x, B.SNN_ACT_BIN_ROWS)
        ws = B.snn_subbit_prepare(d, cb, idx, alpha)
        y = torch.empty((L.N, L.C_out, L.H_out, L.W_out), dtype=torch.float32, device="cuda")
        io.append({"desc": d, "x": xr, "y": y, "workspace": ws})
        del x
    arr = B.layer_io_array(io)
    torch.cuda.synchronize()
    P.copy(b, a)
    torch.cuda.synchronize()
    for _ in range(3):
        B.snn_subbit_conv2d_prepared_many(arr)
        torch.cuda.synchronize()


def run_configs(bn, args, peaks, oracle):
    """Workloads 1-4: microseconds, GOPS-equivalent, speed-up over the 1-bit kernel, roofline, oracle check, cold series."""
    torch, B, np, synth = bn.torch, bn.B, bn.np, bn.synth
    from paper_2110_09195_amd import accounting
    reps = 30
    out = []

    def bin_layer(L, cfg_no, zipf, check_images):
        g = synth.rng(cfg_no, 0)
        s = bn.layer_state(L, g, zipf_w=zipf)
        B.snn_project_kernels(s["w"], s["cb"], out=s["idx"])
        B.snn_pack_activations(s["x"], B.SNN_ACT_BIN_ROWS, out=s["xr"])
        B.snn_pack_activations(s["x"], B.SNN_ACT_BIN_CHANNELS, out=s["xc"])
        idx2 = s["idx"].view(L.C_out, L.C_in)
        B.snn_subbit_prepare(s["d_sub"], s["cb"], idx2, s["alpha"], workspace=s["ws_sub"])
        s["w9"] = s["cb"][s["idx"].long()].view(L.C_out, L.C_in).contiguous()

        def conv():
            B.snn_subbit_conv2d_prepared(s["d_sub"], s["xr"], s["alpha"], s["ws_sub"], y=s["y"])

        def bnn():
            B.snn_bnn_conv2d(s["d_bnn"], s["xc"], s["w9"], s["alpha"], y=s["yb"], workspace=s["ws_bnn"])
        t_conv = bn.event_avg_us(conv, reps)
        each = bn.event_each_us(conv, reps)
        t_bnn = bn.event_avg_us(bnn, reps)
        torch.cuda.synchronize()
        assert torch.equal(s["y"], s["yb"]), "sub-bit and 1-bit kernels disagree on " + L.name
        slots = B.snn_subbit_slots_per_channel(s["d_sub"])
        row = {"layer": L.name, "K": L.K, "index_dist": "zipf(1.1)" if zipf else "uniform",
               "conv_us": t_conv, "conv_us_single_launch_median": each[len(each) // 2], "conv_us_single_launch_min": each[0],
               "conv_us_cold": bn.cold_us(conv), "gops_eq": L.dense_ops / (t_conv * 1e-6) / 1e9,
               "bnn_conv_us": t_bnn, "bnn_conv_us_cold": bn.cold_us(bnn), "speedup_vs_bnn_conv": t_bnn / t_conv,
               "pack_rows_us": bn.event_avg_us(lambda: B.snn_pack_activations(s["x"], B.SNN_ACT_BIN_ROWS, out=s["xr"]), reps),
               "project_us": bn.event_avg_us(lambda: B.snn_project_kernels(s["w"], s["cb"], out=s["idx"]), reps),
               "timing": "conv_us / bnn_conv_us: %d launches back to back between one pair of HIP events; single_launch: one "
                         "pair per launch; cold: 512 MB written between launches, median of 7" % reps}
        if slots > 0:
            rf = conv_roofline([L], [slots], t_conv * 1e-6, peaks, accounting)
            row["roofline"] = {k: rf[k] for k in ("bound", "alg_bytes", "gather_adds", "responses", "slots_per_channel", "frac",
                                                   "frac_hbm", "frac_unit", "useful_frac", "frac_vs_measured_peaks") if k in rf}
        if oracle is not None:
            n = min(check_images, L.N)
            idx_o, _ = oracle.project(s["w"].cpu().numpy(), s["cb"].cpu().numpy().view(np.uint16))
            assert (idx_o.reshape(-1) == s["idx"].cpu().numpy().view(np.uint16)).all(), "projection differs from the oracle on " + L.name
            c0 = time.perf_counter()
            _, Y = oracle.conv_bin(oracle.sign(s["x"][:n].cpu().numpy()), oracle.expand(s["cb"].cpu().numpy().view(np.uint16), idx_o.reshape(L.C_out, L.C_in)),
                                   s["alpha"].cpu().numpy(), L.stride)
            row["oracle_s"] = time.perf_counter() - c0
            assert (s["y"][:n].cpu().numpy() == Y).all(), "GPU result differs from the oracle on " + L.name
            row["checked"] = "indices of all kernels and outputs of the first %d images equal the oracle's, bit for bit" % n
        return s, row

    # ---- config 1 ----
    s, row = bin_layer(synth.CFG1, 1, False, synth.CFG1.N)
    row["config"] = 1
    row["note"] = "a few microseconds of work: bound by launch latency"
    out.append(row)

    # ---- config 2: fp32 activations ----
    L = synth.CFG2
    g = synth.rng(2, 0)
    x = bn.dev(synth.activations(g, L.N, L.C_in, L.H, L.W))
    cb = bn.dev(synth.codebook(g, L.K))
    idx = bn.dev(synth.indices(g, L.C_out, L.C_in, L.K))
    alpha = bn.dev(synth.alpha(g, L.C_out))
    d = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_F32)
    y = torch.empty((L.N, L.C_out, L.H_out, L.W_out), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(d, B.SNN_WS_SUBBIT)

    def conv_f32():
        B.snn_subbit_conv2d(d, x, cb, idx, alpha, y=y, workspace=ws)
    t = bn.event_avg_us(conv_f32, reps)
    each = bn.event_each_us(conv_f32, reps)
    lane_ops = accounting.stage1_responses(L) * 9 + accounting.stage2_gather_adds(L)
    alg_bytes = L.N * L.C_in * L.H * L.W * 4 + L.pixels * L.C_out * 4 + L.C_in * L.C_out * 2
    row = {"config": 2, "layer": L.name, "K": L.K, "activations": "fp32", "conv_us": t,
           "conv_us_single_launch_median": each[len(each) // 2], "conv_us_cold": bn.cold_us(conv_f32),
           "gops_eq": L.dense_ops / (t * 1e-6) / 1e9,
           "roofline": {"bound": "alu", "alg_bytes": alg_bytes, "responses": accounting.stage1_responses(L),
                        "gather_adds": accounting.stage2_gather_adds(L),
                        "unit_used": "plain fp32 VALU adds: 9 per response, 1 per gather-add",
                        "frac": max(alg_bytes / HBM_PEAK_BYTES, lane_ops / VALU_PEAK_LANE_OPS) / (t * 1e-6),
                        "frac_hbm": alg_bytes / HBM_PEAK_BYTES / (t * 1e-6), "frac_unit": lane_ops / VALU_PEAK_LANE_OPS / (t * 1e-6)},
           "note": "the call includes its small table-preparation kernel; a few microseconds of work: bound by launch latency"}
    if oracle is not None:
        _, Y = oracle.conv_f32(x.cpu().numpy(), oracle.expand(cb.cpu().numpy().view(np.uint16), idx.cpu().numpy().view(np.uint16)),
                               alpha.cpu().numpy(), L.stride)
        got = y.cpu().numpy().astype(np.float64)
        denom = np.maximum(np.abs(Y), np.sqrt(np.mean(np.square(Y.astype(np.float64)))))
        err = float(np.max(np.abs(got - Y) / denom))
        assert err <= 1e-5, "fp32-activation result differs from the oracle: %.3g" % err
        row["checked"] = "every output within 1e-5 * max(|ref|, rms(ref)) of the fp64 oracle (largest: %.2e)" % err
    out.append(row)
    del x, y

    # ---- config 3: Zipf indices; the 1-bit kernel on the same weights and on uniform codes; identity-512 ----
    L = synth.CFG3
    s, row = bin_layer(L, 3, True, 8)
    row["config"] = 3
    g = synth.rng(3, 50)
    w9u = bn.dev(g.integers(0, 512, size=(L.C_out, L.C_in)).astype(np.uint16))

    def bnn_uniform():
        B.snn_bnn_conv2d(s["d_bnn"], s["xc"], w9u, s["alpha"], y=s["yb"], workspace=s["ws_bnn"])
    row["bnn_conv_us_uniform_w9"] = bn.event_avg_us(bnn_uniform, reps)
    row["bnn_conv_us_same_weights"] = row["bnn_conv_us"]
    # the 1-bit layer through the sub-bit path: identity subset of all 512 kernels, idx = the kernel codes (an invariant
    # check, Sec. 4.1: a 1-bit layer is the sub-bit layer whose subset is the whole set; runs on the LDS-gather kernel)
    d512 = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, 512, B.SNN_ACT_BIN_ROWS)
    ident = bn.dev(np.arange(512, dtype=np.uint16))
    ws512 = B.alloc_workspace(d512, B.SNN_WS_SUBBIT)
    y512 = torch.empty_like(s["y"])

    def conv512():
        B.snn_subbit_conv2d(d512, s["xr"], ident, w9u, s["alpha"], y=y512, workspace=ws512)
    row["subbit_identity512_us"] = bn.event_avg_us(conv512, reps)
    torch.cuda.synchronize()
    assert torch.equal(y512, s["yb"]), "identity-512 sub-bit layer and 1-bit kernel disagree"
    row["identity512_note"] = "labelled invariant run, not the baseline: equals snn_bnn_conv2d on the same uniform codes, bit for bit"
    out.append(row)
    del s, y512

    # ---- config 4: K sweep ----
    for K in (16, 32, 64):
        s, row = bin_layer(synth.cfg4(K), 4, False, 4)
        row["config"] = 4
        out.append(row)
        del s
    torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over the batch without communication); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.counter_child:
        counter_child(args)
        return

    # the counter passes are child processes of their own and run before this process touches the GPU
    traffic = None
    if not (args.no_traffic or args.headline_only):
        traffic = measure_traffic(args)

    import numpy as np
    import torch

    from paper_2110_09195_amd import accounting, synth
    from paper_2110_09195_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    B.lib()
    bn = Bench(torch, B, np, synth)
    dev = bn.dev
    oracle = None
    if not args.no_cpu:
        import oracle
        oracle.build()

    layers, wname, cfg_no = workload_of(args, synth)
    extras = not args.headline_only

    # ---- resident inputs and buffers -------------------------------------------------------------
    st = [bn.layer_state(L, synth.rng(cfg_no, i), zipf_w=(args.workload == "cfg3" and not args.layer),
                         extra=("forward", "dense")) for i, L in enumerate(layers)]
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

    def conv_prepared(s):
        B.snn_subbit_conv2d_prepared(s["d_sub"], s["xr"], s["alpha"], s["ws_sub"], y=s["y"])

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

    # The headline step, three launches: sign/pack of all layers' inputs, the weights-side work of all layers (projection +
    # tables), the convolutions of all layers.  For the roofline the same steps run a second time with a pair of events
    # on the launch stream around the convolution launch: their average is the kernel time it uses.
    prep_arr = B.layer_weights_array([{"desc": s["d_sub"], "w": s["w"], "codebook": s["cb"], "alpha": s["alpha"],
                                       "idx_out": s["idx"], "workspace": s["ws_sub"]} for s in st])
    many_ok = all(B.snn_subbit_slots_per_channel(s["d_sub"]) > 0 for s in st)
    io_arr = B.layer_io_array([{"desc": s["d_sub"], "x": s["xr"], "y": s["y"], "workspace": s["ws_sub"]} for s in st]) if many_ok else None
    ev = []

    def convs():
        if many_ok:
            B.snn_subbit_conv2d_prepared_many(io_arr)
        else:
            for s in st:
                conv_prepared(s)

    # the same step as ONE call (snn_subbit_forward_many: the same three launches; its own workspaces and outputs)
    fwd_many = None
    if many_ok:
        fwd_arr = B.layer_forward_array([{"desc": s["d_sub"], "x": s["x"], "w": s["w"], "codebook": s["cb"], "alpha": s["alpha"],
                                          "idx_out": s["idx"], "y": s["y"], "workspace": s["ws_fwd"]} for s in st])

        def fwd_many():
            B.snn_subbit_forward_many(fwd_arr)

    pack_arr = B.pack_item_array([(s["x"], s["xr"], B.SNN_ACT_BIN_ROWS) for s in st])

    def step(timed=False):
        if not timed and fwd_many is not None:
            fwd_many()                      # the same three launches as one call
            return
        B.snn_pack_activations_many(pack_arr)
        B.snn_subbit_project_prepare_many(prep_arr)
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            convs()
            e1.record()
            ev.append((e0, e1))
        else:
            convs()

    def step_per_layer_launches():
        B.snn_subbit_project_prepare_many(prep_arr)
        for s in st:
            pack_rows(s)
            conv_prepared(s)

    def step_pack_per_layer():
        B.snn_subbit_project_prepare_many(prep_arr)
        for s in st:
            pack_rows(s)
        convs()

    def step_forward_calls():
        for s in st:
            forward(s)

    def step_separate():
        for s in st:
            project(s)
            pack_rows(s)
            conv_sub(s)

    def conv_bnn_prepared(s):
        B.snn_bnn_conv2d_prepared(s["d_bnn"], s["xc"], s["alpha"], s["ws_bnn"], y=s["yb"])

    def step_bnn():
        for s in st:
            pack_channels(s)
            conv_bnn(s)

    def step_inference():
        B.snn_pack_activations_many(pack_arr)
        convs()

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
    # the same K steps once more with a pair of HIP events around the convolution launch of every step (kept out of
    # the region above: an event pair costs the step some 15 us)
    for _ in range(args.steps):
        step(timed=True)
    torch.cuda.synchronize()
    in_step = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    t_conv_in_step_us = sum(in_step) / len(in_step)

    ms_per_step_bnn = bn.host_ms(step_bnn, args.warmup, args.steps)
    ms_per_step_per_layer = bn.host_ms(step_per_layer_launches, args.warmup, args.steps)
    ms_per_step_pack_per_layer = bn.host_ms(step_pack_per_layer, args.warmup, args.steps)
    ms_per_step_three_calls = None
    if fwd_many is not None:
        def three_calls():
            B.snn_pack_activations_many(pack_arr)
            B.snn_subbit_project_prepare_many(prep_arr)
            convs()
        ms_per_step_three_calls = bn.host_ms(three_calls, args.warmup, args.steps)
        torch.cuda.synchronize()
        want = [(s["y"].clone(), s["idx"].clone()) for s in st]
        for s in st:
            s["y"].fill_(float("nan"))
        fwd_many()
        torch.cuda.synchronize()
        for s, (y3, i3) in zip(st, want):
            assert torch.equal(s["y"], y3) and torch.equal(s["idx"], i3), "forward_many differs from the three calls on " + s["L"].name
        del want
    ms_per_step_inference = bn.host_ms(step_inference, args.warmup, args.steps)
    ms_per_step_forward_calls = ms_per_step_separate = ms_per_step_dense = ms_per_step_dense_inference = None
    if extras:
        ms_per_step_forward_calls = bn.host_ms(step_forward_calls, args.warmup, args.steps)
        ms_per_step_separate = bn.host_ms(step_separate, args.warmup, args.steps)
        ms_per_step_dense = bn.host_ms(step_dense, args.warmup, args.steps)
        ms_per_step_dense_inference = bn.host_ms(step_dense_inference, args.warmup, args.steps)

    # ---- the same stack as a chain of 1-bit activations (resnet18 workload only) ---------------------------
    # Layer i's convolution ends in the next layer's binarisation (snn_subbit_forward_sign): the packed output of one
    # layer is the packed input of the next, no fp32 activations are written and nothing is packed in between.
    # Reported next to the headline, not as it: the headline's layers each take their own fp32 input.
    chained = None
    chain_ok = extras and args.workload == "resnet18" and not args.layer and all(
        a.C_out == b.C_in and a.H_out == b.H and a.W_out == b.W for a, b in zip(layers, layers[1:]))
    if chain_ok:
        for i, s in enumerate(st):
            L = s["L"]
            s["beta"] = dev((0.25 * synth.rng(cfg_no, 200 + i).standard_normal(L.C_out)).astype(np.float32))
            words = L.N * L.C_out * L.H_out * ((L.W_out + 31) // 32)
            s["out_bits"] = torch.empty(words, dtype=torch.int32, device="cuda")
            s["ws_chain"] = B.alloc_workspace(s["d_sub"], B.SNN_WS_SUBBIT)
        chain_arr = B.layer_weights_array([{"desc": s["d_sub"], "w": s["w"], "codebook": s["cb"], "alpha": s["alpha"],
                                            "beta": s["beta"], "idx_out": s["idx"], "workspace": s["ws_chain"]} for s in st])

        def step_chained():
            B.snn_subbit_project_prepare_many(chain_arr)
            xin = B.snn_pack_activations(st[0]["x"], B.SNN_ACT_BIN_ROWS, out=st[0]["xr"])
            for s in st:
                B.snn_subbit_conv2d_sign_prepared(s["d_sub"], xin, s["ws_chain"], out=s["out_bits"])
                xin = s["out_bits"]
        ms_chained = bn.host_ms(step_chained, args.warmup, args.steps)
        for s in st:
            L = s["L"]
            s["ws_sign"] = B.snn_subbit_prepare_sign(s["d_sub"], s["cb"], s["idx"].view(L.C_out, L.C_in), s["alpha"], s["beta"])

        def step_chained_inference():
            xin = B.snn_pack_activations(st[0]["x"], B.SNN_ACT_BIN_ROWS, out=st[0]["xr"])
            for s in st:
                B.snn_subbit_conv2d_sign_prepared(s["d_sub"], xin, s["ws_sign"], out=s["out_bits"])
                xin = s["out_bits"]
        ms_chained_inf = bn.host_ms(step_chained_inference, args.warmup, args.steps)
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
        ms_chained_dense = bn.host_ms(step_chained_dense, args.warmup, args.steps)
        chained = {"ms_per_step": ms_chained, "gops_eq": sum(L.dense_ops for L in layers) / (ms_chained * 1e-3) / 1e9,
                   "ms_per_step_inference_dense_context": ms_chained_dense,
                   "ms_per_step_inference": ms_chained_inf,
                   "inference_step": "weights prepared once (snn_subbit_prepare_sign); pack the first input, then one "
                                     "snn_subbit_conv2d_sign_prepared launch per layer",
                   "step": "snn_subbit_project_prepare_many (projection + thresholds + tables of all layers), pack the first "
                           "input, then one snn_subbit_conv2d_sign_prepared per layer: 1-bit activations from layer to layer"}

    # the yardsticks (after the timed regions: the matrix probes heat the chip, and what runs right after them
    # runs at a lower clock for a while)
    peaks = measured_peaks(torch, np)

    # ---- per-call device time with HIP events on the launch stream ---------------------------------------
    reps = max(10, min(args.steps, 30))
    # restore what the steps above may have left in the buffers the checks read
    step()
    for s in st:
        pack_channels(s)
        conv_bnn(s)
    torch.cuda.synchronize()
    # the two kernels must agree (same decoded weights): a cheap end-to-end sanity check
    for s in st:
        assert torch.equal(s["y"], s["yb"]), "sub-bit and 1-bit kernels disagree on " + s["L"].name

    t_convs_b2b = bn.event_avg_us(convs, reps)                     # the convolution launch, back to back
    t_convs_each = bn.event_each_us(convs, reps)
    t_convs_cold = bn.cold_us(convs)
    t_prep_many = bn.event_avg_us(lambda: B.snn_subbit_project_prepare_many(prep_arr), reps)
    t_pack_many = bn.event_avg_us(lambda: B.snn_pack_activations_many(pack_arr), reps)
    t_kern = [bn.event_avg_us(lambda s=s: conv_prepared(s), reps) for s in st]      # one launch per layer, for comparison
    t_bnn = [bn.event_avg_us(lambda s=s: conv_bnn(s), reps) for s in st]
    # the same 1-bit convolutions from prepared weights (the workspaces hold them since conv_bnn above): the form to
    # set beside the sub-bit launch, which also starts from prepared tables
    t_bnn_k = [bn.event_avg_us(lambda s=s: conv_bnn_prepared(s), reps) for s in st]
    for s in st:
        assert torch.equal(s["y"], s["yb"]), "prepared 1-bit kernel disagrees on " + s["L"].name
    # XOR + bit count: 2 lane-operations per 32-bit word of a tap (Sec. 3), 9 ceil(C_in / 32) words per output
    bnn_lane_ops = sum(2 * 9 * ((L.C_in + 31) // 32) * L.N * L.H_out * L.W_out * L.C_out for L in layers)
    t_proj = [bn.event_avg_us(lambda s=s: project(s), reps) for s in st]
    t_pr = [bn.event_avg_us(lambda s=s: pack_rows(s), reps) for s in st]
    t_pc = [bn.event_avg_us(lambda s=s: pack_channels(s), reps) for s in st]
    t_bnn_cold = sum(bn.cold_us(lambda s=s: conv_bnn(s), 5) for s in st)
    t_dense = t_dense_k = None
    if extras:
        t_dense = [bn.event_avg_us(lambda s=s: conv_dense(s), reps) for s in st]
        t_dense_k = [bn.event_avg_us(lambda s=s: conv_dense_prepared(s), reps) for s in st]

    # training-side lines of Alg. 1 (not part of the step, which is the forward pass)
    training = None
    if extras:
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
        t_pb = [bn.event_avg_us(lambda s=s: B.snn_project_backward(s["w"], s["g_wbar"], s["idx"], s["L"].K, g_w=s["g_w"],
                                                                  g_p=s["g_p"], workspace=s["ws_bwd"]), reps) for s in st]
        t_su = [bn.event_avg_us(lambda s=s: B.snn_subset_update(s["p"], s["m"], 1e-3), reps) for s in st]
        bwd_bytes = sum(L.C_out * L.C_in * (36 + 36 + 2 + 36) for L in layers)
        training = {"project_backward_us": sum(t_pb), "subset_update_us": sum(t_su),
                    "project_backward_GBps": bwd_bytes / (sum(t_pb) * 1e-6) / 1e9,
                    "note": "launches back to back between one pair of events, summed over the layers; Alg. 1 backward lines, "
                            "outside the step"}

    # 1x1 layers of a bottleneck network (appendix, Table 5): shapes of ResNet-50 at batch 64, K = 32 members of {+-1}^8
    conv1x1 = None
    if extras and args.workload == "resnet18" and not args.layer:
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
            us = bn.event_avg_us(lambda: B.snn_subbit_conv1x1(d1, x1, cb1, idx1, al1, y=y1, workspace=ws1), reps)
            B.snn_subbit_conv1x1_prepare(d1, cb1, idx1, al1, workspace=ws1)
            us_p = bn.event_avg_us(lambda: B.snn_subbit_conv1x1_prepared(d1, x1, ws1, y=y1), reps)
            ops = 2.0 * ci * co * 64 * hw * hw
            conv1x1.append({"layer": "%d->%d %dx%d" % (ci, co, hw, hw), "us": us, "prepared_us": us_p,
                            "gops_eq_prepared": ops / (us_p * 1e-6) / 1e9,
                            "out_GBps_prepared": 64 * co * hw * hw * 4 / (us_p * 1e-6) / 1e9})
            del x1, y1

    dense_ops = sum(L.dense_ops for L in layers)
    in_bytes_packed = sum(L.N * L.C_in * L.H * ((L.W + 31) // 32) * 4 for L in layers)
    slots = [B.snn_subbit_slots_per_channel(s["d_sub"]) for s in st]
    roofline = None
    if many_ok:
        roofline = conv_roofline(layers, slots, t_conv_in_step_us * 1e-6, peaks, accounting)
        roofline["kernel"] = ("subbit_stack_kernel: ONE launch per step runs the convolutions of all %d layers (resident workers of "
                              "one wave draw (layer, tile) items); t_kernel = average over %d steps (the timed steps run a second time) of a "
                              "HIP-event pair around that launch, on the launch stream" % (len(layers), args.steps))
        roofline["t_kernel_us_back_to_back"] = t_convs_b2b
        roofline["t_kernel_us_single_launch_median"] = t_convs_each[len(t_convs_each) // 2]
        roofline["t_kernel_us_single_launch_min"] = t_convs_each[0]
        roofline["t_kernel_us_cold"] = t_convs_cold
        roofline["t_kernel_us_in_step_min_max"] = [in_step[0], in_step[-1]]
        roofline["traffic"] = traffic
        if traffic:
            roofline["traffic_over_alg_bytes"] = traffic["bytes"] / roofline["alg_bytes"]
        roofline["peaks_vendor"] = {"hbm_GBps": HBM_PEAK_BYTES / 1e9, "mfma_fp6_fp4_TFLOPs": MFMA_FP6_FP4_PEAK_FLOPS / 1e12,
                                    "valu_T_lane_ops": VALU_PEAK_LANE_OPS / 1e12}
        roofline["peaks_measured"] = peaks

    print("%-18s %9s %6s %5s | %9s %9s %7s | %8s %8s %8s" % ("layer", "pixels", "C", "K", "subbit us", "bnn us", "ratio",
                                                             "proj us", "packR us", "packC us"), file=sys.stderr)
    for L, a, b, c, d, e in zip(layers, t_kern, t_bnn, t_proj, t_pr, t_pc):
        print("%-18s %9d %3d>%-3d %4d | %9.1f %9.1f %7.2f | %8.1f %8.1f %8.1f" % (
            L.name, L.pixels, L.C_in, L.C_out, L.K, a, b, b / a, c, d, e), file=sys.stderr)
    print("sums of per-layer launches: subbit %.1f us, bnn %.1f us, project %.1f us, pack rows %.1f us, pack channels %.1f us"
          % (sum(t_kern), sum(t_bnn), sum(t_proj), sum(t_pr), sum(t_pc)), file=sys.stderr)
    print("all convolutions in one launch: %.1f us inside the step, %.1f us back to back, %.1f us cold; prepare_many %.1f us; "
          "pack_many %.1f us" % (t_conv_in_step_us, t_convs_b2b, t_convs_cold, t_prep_many, t_pack_many), file=sys.stderr)
    print("step %.1f us (as three calls: %s us; with one pack launch per layer: %.1f us; with one pack and one "
          "convolution launch per layer: %.1f us); inference step %.1f us; 1-bit step %.1f us"
          % (ms_per_step * 1e3, "%.1f" % (ms_per_step_three_calls * 1e3) if ms_per_step_three_calls else "-",
             ms_per_step_pack_per_layer * 1e3, ms_per_step_per_layer * 1e3, ms_per_step_inference * 1e3, ms_per_step_bnn * 1e3),
          file=sys.stderr)
    if extras:
        print("step as one snn_subbit_forward per layer: %.1f us; as three separate calls per layer: %.1f us"
              % (ms_per_step_forward_calls * 1e3, ms_per_step_separate * 1e3), file=sys.stderr)
        print("dense FP4 context: step %.1f us, prepared %.1f us; conv calls %.1f us, prepared %.1f us"
              % (ms_per_step_dense * 1e3, ms_per_step_dense_inference * 1e3, sum(t_dense), sum(t_dense_k)), file=sys.stderr)
    if chained is not None:
        print("chained 1-bit stack: %.1f us; prepared weights: %.1f us; through the dense contraction (prepared): %.1f us"
              % (chained["ms_per_step"] * 1e3, chained["ms_per_step_inference"] * 1e3,
                 chained["ms_per_step_inference_dense_context"] * 1e3), file=sys.stderr)

    # ---- the other workloads -------------------------------------------------------------------------------
    configs = None
    if extras and not args.no_configs and args.workload == "resnet18" and not args.layer:
        configs = run_configs(bn, args, peaks, oracle)
        for r in configs:
            print("config %d %-22s K=%-3d conv %8.1f us (cold %8.1f)  %9.0f GOPS-eq  vs 1-bit %s  frac %s" % (
                r["config"], r["layer"], r["K"], r["conv_us"], r["conv_us_cold"], r["gops_eq"],
                "%.2fx" % r["speedup_vs_bnn_conv"] if "speedup_vs_bnn_conv" in r else "  -  ",
                "%.2f" % r["roofline"]["frac"] if "roofline" in r else "-"), file=sys.stderr)

    # ---- cpu_baseline: the oracle on a bounded sample of the same workload --------------------------------
    cpu = None
    if oracle is not None:
        # refresh the headline outputs (the extra legs share buffers)
        step()
        torch.cuda.synchronize()
        n_img = 64 if args.workload == "resnet18" else 16
        t_cpu = 0.0
        ops_cpu = 0
        for s in st:
            L = s["L"]
            n = min(n_img, L.N)
            x = s["x"][:n].cpu().numpy()
            w = s["w"].cpu().numpy()
            cb = s["cb"].cpu().numpy().view(np.uint16)
            alpha = s["alpha"].cpu().numpy()
            c0 = time.perf_counter()
            idx, _ = oracle.project(w, cb)
            xs = oracle.sign(x)
            _, Y = oracle.conv_bin(xs, oracle.expand(cb, idx.reshape(L.C_out, L.C_in)), alpha, L.stride)
            t_cpu += time.perf_counter() - c0
            ops_cpu += L.dense_ops // L.N * n
            assert (idx.reshape(-1) == s["idx"].cpu().numpy().view(np.uint16)).all(), "projection differs from the oracle on " + L.name
            assert (s["y"][:n].cpu().numpy() == Y).all(), "GPU result differs from the oracle on " + L.name
        if chained is not None:
            # the chain, first two images, layer by layer against the oracle (images are independent)
            step_chained()
            step_chained_dense()
            torch.cuda.synchronize()
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
               "sample": "same %d layers, all kernels projected, first %d images of the batch (project + sign + direct conv), "
                         "%.1f s; the GPU's indices and those images' outputs equal the oracle's bit for bit" % (
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
        "dtype": "fp4 x fp6 -> f32 (exact integers; one f32 multiply by alpha)",
        "data": "synthetic",
        "config": {"workload": wname,
                   "step": "one snn_subbit_forward_many call = three launches: sign + pack of all layers' inputs "
                           "(snn_pack_activations_many), projection + tables of all layers (snn_subbit_project_prepare_many), "
                           "the convolutions of all layers (snn_subbit_conv2d_prepared_many)" if many_ok else
                           "snn_subbit_project_prepare_many, then per layer snn_pack_activations + snn_subbit_conv2d_prepared"},
        "ms_per_step_three_calls": ms_per_step_three_calls,
        "ms_per_step_pack_launch_per_layer": ms_per_step_pack_per_layer,
        "ms_per_step_pack_and_conv_launch_per_layer": ms_per_step_per_layer,
        "ms_per_step_forward_calls": ms_per_step_forward_calls,
        "ms_per_step_separate_calls": ms_per_step_separate,
        "ms_per_step_inference": ms_per_step_inference,
        "inference_step": "weights prepared once; snn_pack_activations_many + the convolution launch",
        "conv_us_in_step": t_conv_in_step_us,
        "conv_only_gops_eq": dense_ops / (t_conv_in_step_us * 1e-6) / 1e9,
        "conv_kernel_us_per_layer_launches": t_kern,
        "bnn_conv_us_per_layer": t_bnn,
        "bnn_conv_only_gops_eq": dense_ops / (sum(t_bnn) * 1e-6) / 1e9,
        "speedup_vs_bnn_conv": sum(t_bnn) / t_conv_in_step_us,
        "bnn_conv_prepared_us_per_layer": t_bnn_k,
        "speedup_vs_bnn_conv_prepared": sum(t_bnn_k) / t_conv_in_step_us,
        "bnn_roofline": {"bound": "alu", "kernel": "bnn_regs_kernel (snn_bnn_conv2d_prepared, sixteen launches)",
                         "lane_ops": bnn_lane_ops, "us": sum(t_bnn_k),
                         "achieved": bnn_lane_ops / (sum(t_bnn_k) * 1e-6) / 1e12, "unit": "T lane-op/s",
                         "peak": VALU_PEAK_LANE_OPS / 1e12, "frac": bnn_lane_ops / VALU_PEAK_LANE_OPS / (sum(t_bnn_k) * 1e-6),
                         "frac_vs_measured_xor_bcnt": bnn_lane_ops / (peaks["valu_xor_bcnt_T_lane_ops"] * 1e12) / (sum(t_bnn_k) * 1e-6)},
        "speedup_vs_bnn_conv_cold": t_bnn_cold / t_convs_cold,
        "speedup_vs_bnn_step": ms_per_step_bnn / ms_per_step,
        "bnn_ms_per_step": ms_per_step_bnn,
        "breakdown_us": {"subbit_conv_one_launch": t_conv_in_step_us, "subbit_conv_per_layer_launches": sum(t_kern),
                         "project_prepare_many": t_prep_many, "pack_many": t_pack_many, "bnn_conv": sum(t_bnn), "project": sum(t_proj),
                         "pack_rows": sum(t_pr), "pack_channels": sum(t_pc)},
        "other_step_kernels": {
            "pack_rows_many_kernel": {
                "us": t_pack_many, "alg_bytes": sum(L.N * L.C_in * L.H * L.W * 4 for L in layers) + in_bytes_packed,
                "bound": "hbm",
                "frac": (sum(L.N * L.C_in * L.H * L.W * 4 for L in layers) + in_bytes_packed) / HBM_PEAK_BYTES / (t_pack_many * 1e-6),
                "frac_vs_measured_read": (sum(L.N * L.C_in * L.H * L.W * 4 for L in layers) + in_bytes_packed)
                / (peaks["hbm_read_GBps"] * 1e9) / (t_pack_many * 1e-6)},
            "subbit_prepare_many_kernel": {
                "us": t_prep_many, "alg_bytes": sum(L.C_in * L.C_out * 38 for L in layers),
                "lane_ops": sum(L.C_in * L.C_out * L.K * 10 for L in layers), "bound": "alu",
                "frac": max(sum(L.C_in * L.C_out * 38 for L in layers) / HBM_PEAK_BYTES,
                            sum(L.C_in * L.C_out * L.K * 10 for L in layers) / VALU_PEAK_LANE_OPS) / (t_prep_many * 1e-6),
                "frac_hbm": sum(L.C_in * L.C_out * 38 for L in layers) / HBM_PEAK_BYTES / (t_prep_many * 1e-6),
                "note": "Eq. 2 / Eq. 5: per kernel and subset member nine sequential fp32 add/subtracts and one comparison "
                        "(10 lane-operations; 36 bytes in and 2 out per kernel).  As built a member costs 12 vector "
                        "instructions (the comparison is a compare and two selects), and the selector words, tables and "
                        "ballots of the block come on top: the launch is bound by vector issue at five waves per SIMD"}},
        "training_side": training,
        "chained_1bit_stack": chained,
        "dense_fp4_context": None if not extras else {
            "what": "the same sub-bit layers (subset + indices) through snn_subbit_conv2d_dense: kernels looked up and "
                    "expanded by a preparation kernel, then a dense FP4 contraction on the matrix cores without the "
                    "sharing of Sec. 4.5; context, not the paper's method",
            "ms_per_step": ms_per_step_dense, "ms_per_step_inference": ms_per_step_dense_inference,
            "conv_us": sum(t_dense), "conv_prepared_us": sum(t_dense_k),
            "conv_prepared_us_per_layer": t_dense_k,
            "subbit_over_dense_conv_prepared": t_conv_in_step_us / sum(t_dense_k)},
        "conv1x1_resnet50_shapes": conv1x1,
        "configs": configs,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
