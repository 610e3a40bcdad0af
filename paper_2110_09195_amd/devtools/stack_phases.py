"""Where the time of the one-launch convolution stack goes: wall-clock marks inside the kernel.

    python -m paper_2110_09195_amd.devtools.stack_phases build      # anywhere: hipcc cross-compiles
    python -m paper_2110_09195_amd.devtools.stack_phases run        # on the GPU

`build` writes an INSTRUMENTED COPY of csrc/subbit_stack.hip to a temporary directory (the product source and
library are not touched and carry no trace code), compiles it with the other sources into
devtools/libsnn_hip_phases.so, and `run` loads that library, launches the ResNet-18 stack (batch 64, K = 32) once
warm, and summarises the marks: per layer the mean duration of a tile's phases (run lookup, set-up, pipeline fill,
loop, finishing step), the loop's clocks per matrix instruction and wave, how much of the launch a SIMD has one or
two waves resident / in their loops, and a time line of the workers' states.  Every item (layer, tile) writes 16
words into a buffer whose device address the instrumented launcher reads from the environment variable
SNN_TRACE_PTR; lane 0 writes them with plain vector stores.

The instrumentation is a list of exact text substitutions: if the kernel source changes under one of them the build
stops with the missing anchor instead of producing a half-instrumented kernel.
"""
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsnn_hip_phases.so")

# (anchor, replacement, every occurrence?)
SUBSTITUTIONS = [
    ('#include <algorithm>\n', '#include <algorithm>\n#include <stdlib.h>\n', False),
    ('    int n_tail;               // the last n_tail items',
     '    unsigned long long *trace;\n    int n_tail;               // the last n_tail items', False),
    ('template <int... I, typename F>',
     '#define ST_MARK(i) do { if (threadIdx.x == 0) trow[(i)] = wall_clock64(); } while (0)\ntemplate <int... I, typename F>', False),
    ('uint32_t *const sched, uint32_t &drawn)\n{',
     'uint32_t *const sched, uint32_t &drawn, unsigned long long *const trow)\n{', False),
    ('    constexpr bool ONE_WORD = WM == 1 || STG;',
     '    ST_MARK(2);\n    constexpr bool ONE_WORD = WM == 1 || STG;', False),
    ('    int c = 0;\n    if (UNROLL <= c_end) {\n',
     '    ST_MARK(3);\n    if (threadIdx.x == 0) trow[11] = clock64();\n    int c = 0;\n    if (UNROLL <= c_end) {\n', False),
    ('    if (c < c_end) group(c, std::true_type{}, std::false_type{});\n',
     '    if (c < c_end) group(c, std::true_type{}, std::false_type{});\n    ST_MARK(4);\n'
     '    if (threadIdx.x == 0) trow[12] = clock64();\n', False),
    ('        const u32x2 run = *(lds_cu32x2 *)',
     '        unsigned long long *const trow = sp.trace + (size_t)item * 16;\n        ST_MARK(0);\n'
     '        const u32x2 run = *(lds_cu32x2 *)', False),
    ('        const StackLayer &L = sp.layer[l];\n',
     '        const StackLayer &L = sp.layer[l];\n        if (lane == 0) {\n'
     '            trow[8] = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));      // HW_ID\n'
     '            trow[9] = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (31 << 11));     // XCC_ID\n'
     '            trow[10] = (unsigned long long)l;\n        }\n        ST_MARK(1);\n', False),
    ('new_layer, counter, drawn); break;', 'new_layer, counter, drawn, trow); break;', True),
    ('        asm volatile("s_waitcnt vmcnt(0)" : "+v"(drawn) : : "memory");\n',
     '        asm volatile("s_waitcnt vmcnt(0)" : "+v"(drawn) : : "memory");\n        ST_MARK(7);\n', False),
    ('    hipLaunchKernelGGL(subbit_stack_kernel, dim3((unsigned)sp.n_workers)',
     '    sp.trace = (unsigned long long *)strtoull(getenv("SNN_TRACE_PTR") ? getenv("SNN_TRACE_PTR") : "0", nullptr, 0);\n'
     '    if (!sp.trace) return SNN_ERR_INVALID_ARG;\n'
     '    hipLaunchKernelGGL(subbit_stack_kernel, dim3((unsigned)sp.n_workers)', False),
]


def instrumented_source():
    src = open(os.path.join(PKG, "csrc", "subbit_stack.hip")).read()
    for anchor, replacement, every in SUBSTITUTIONS:
        if anchor not in src:
            raise SystemExit("stack_phases: the kernel source no longer contains the anchor\n" + anchor)
        src = src.replace(anchor, replacement) if every else src.replace(anchor, replacement, 1)
    return src


def build():
    from paper_2110_09195_amd import build as B
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory(prefix="snn_phases_") as tmp:
        path = os.path.join(tmp, "subbit_stack.hip")
        open(path, "w").write(instrumented_source())
        objs = []
        for src in B.SOURCES:
            obj = os.path.join(tmp, src + ".o")
            subprocess.run([hipcc] + B.FLAGS + ["-c", path if src == "subbit_stack.hip" else os.path.join(B.CSRC, src), "-o", obj],
                           check=True)
            objs.append(obj)
        subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + objs + ["-o", LIB], check=True)
    print("built", LIB)


def run():
    import numpy as np
    import torch
    from paper_2110_09195_amd import synth, binding as B
    if not os.path.exists(LIB):
        raise SystemExit("stack_phases: build first (python -m paper_2110_09195_amd.devtools.stack_phases build)")
    B.LIB_PATH = LIB
    torch.cuda.set_device(0)
    layers = synth.resnet18_stack(N=64, K=32)

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).cuda()

    st = []
    for i, L in enumerate(layers):
        g = synth.rng(5, i)
        s = {"L": L}
        s["x"] = dev(synth.activations(g, L.N, L.C_in, L.H, L.W))
        s["cb"] = dev(synth.codebook(g, L.K))
        s["w"] = dev(synth.real_kernels(g, L.C_out * L.C_in).astype(np.float32))
        s["alpha"] = dev(synth.alpha(g, L.C_out))
        s["idx"] = torch.empty(L.C_out * L.C_in, dtype=torch.int16, device="cuda")
        s["d"] = B.make_desc(L.N, L.C_in, L.C_out, L.H, L.W, L.stride, L.K, B.SNN_ACT_BIN_ROWS)
        s["xr"] = B.snn_pack_activations(s["x"], B.SNN_ACT_BIN_ROWS)
        s["y"] = torch.zeros((L.N, L.C_out, L.H_out, L.W_out), dtype=torch.float32, device="cuda")
        s["ws"] = B.alloc_workspace(s["d"], B.SNN_WS_SUBBIT)
        st.append(s)
    prep = B.layer_weights_array([{"desc": s["d"], "w": s["w"], "codebook": s["cb"], "alpha": s["alpha"],
                                   "idx_out": s["idx"], "workspace": s["ws"]} for s in st])
    B.snn_subbit_project_prepare_many(prep)
    io = B.layer_io_array([{"desc": s["d"], "x": s["xr"], "y": s["y"], "workspace": s["ws"]} for s in st])
    trace_buf = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    os.environ["SNN_TRACE_PTR"] = str(trace_buf.data_ptr())
    for _ in range(100):                         # the clocks settle after some tens of launches
        B.snn_subbit_conv2d_prepared_many(io)
    torch.cuda.synchronize()
    trace_buf.zero_()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    B.snn_subbit_conv2d_prepared_many(io)
    e1.record()
    torch.cuda.synchronize()
    T = e0.elapsed_time(e1) * 1e3
    tr = trace_buf.cpu().numpy().view(np.uint64).reshape(-1, 16)
    tr = tr[tr[:, 7] != 0]
    t = tr[:, [0, 1, 2, 3, 4, 7]].astype(np.float64) * 0.01          # the wall clock ticks at 100 MHz
    t -= t[:, 0].min()
    span = t[:, 5].max()
    lay = tr[:, 10].astype(int)
    mf = [L.N * L.H_out * L.W_out * L.C_out * L.C_in / 2048.0 for L in layers]     # matrix instructions per layer
    print("one launch between HIP events: %.1f us; first mark to last mark: %.1f us; items %d" % (T, span, len(tr)))
    names = ["lookup", "set-up", "fill", "loop", "finish"]
    print("%-5s %6s %8s | " % ("layer", "tiles", "start") + " ".join("%8s" % n for n in names) + " |   total  instr/tile  clocks/instr")
    cyc = tr[:, 12].astype(np.float64) - tr[:, 11].astype(np.float64)                 # shader clocks inside the loop
    tot = np.zeros(5)
    for l in range(len(layers)):
        m = lay == l
        if not m.any():
            continue
        d = np.diff(t[m], axis=1)
        tot += d.sum(axis=0)
        dm = d.mean(axis=0)
        per_tile = mf[l] / m.sum()
        print("%-5d %6d %8.1f | " % (l, m.sum(), t[m, 0].mean()) + " ".join("%8.2f" % v for v in dm) +
              " | %7.2f  %10.0f  %12.1f" % (dm.sum(), per_tile, np.median(cyc[m]) / per_tile))
    busy = tot.sum()
    print("worker time inside tiles: %.1f us per worker of %.1f (2048 workers): lookup %.1f %%, set-up %.1f %%, fill %.1f %%, "
          "loop %.1f %%, finish %.1f %%" % ((busy / 2048.0, span) + tuple(100.0 * v / busy for v in tot)))
    dur = t[:, 4] - t[:, 3]
    ok = dur > 1.0
    print("shader clock inside the loops: median %.0f MHz (10 %% %.0f, 90 %% %.0f)" % tuple(np.percentile(cyc[ok] / dur[ok], [50, 10, 90])))
    # per SIMD: how long one / two waves are resident, and in their loops
    hw = tr[:, 8].astype(np.int64)
    xcc = tr[:, 9].astype(np.int64) & 15
    key = (((xcc * 8 + ((hw >> 13) & 7)) * 2 + ((hw >> 12) & 1)) * 16 + ((hw >> 8) & 15)) * 4 + ((hw >> 4) & 3)

    def coverage(a, b):
        ev = sorted([(x, 1) for x in a] + [(x, -1) for x in b])
        one = two = 0.0
        n = 0
        last = 0.0
        for x, dlt in ev:
            if n == 1:
                one += x - last
            elif n >= 2:
                two += x - last
            n += dlt
            last = x
        return one / span, two / span

    res, loop = [], []
    for k in np.unique(key):
        m = key == k
        res.append(coverage(t[m, 0], t[m, 5]))
        loop.append(coverage(t[m, 3], t[m, 4]))
    res, loop = np.array(res), np.array(loop)
    print("SIMDs seen: %d; share of the launch with exactly one wave inside a tile %.3f, with two %.3f; with exactly one wave in "
          "its loop %.3f, with two %.3f" % (len(res), res[:, 0].mean(), res[:, 1].mean(), loop[:, 0].mean(), loop[:, 1].mean()))
    total_mf = sum(mf)
    print("matrix instructions %.0f = %.1f per SIMD; at 32 clocks and 2.4 GHz: %.1f us" % (total_mf, total_mf / 1024, total_mf / 1024 * 32 / 2400.0))
    print("time   inside a tile   in the loop   finishing")
    for x in np.linspace(0, span, 21):
        print("%6.1f %10d %12d %12d" % (x, ((t[:, 0] <= x) & (t[:, 5] > x)).sum(), ((t[:, 3] <= x) & (t[:, 4] > x)).sum(),
                                        ((t[:, 4] <= x) & (t[:, 5] > x)).sum()))


if __name__ == "__main__":
    if len(sys.argv) == 2 and sys.argv[1] == "build":
        build()
    elif len(sys.argv) == 2 and sys.argv[1] == "run":
        run()
    else:
        raise SystemExit(__doc__)
