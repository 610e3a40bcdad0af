"""Turn two rocprofv3 --pmc passes (FETCH_SIZE, then WRITE_SIZE; CSV output) of
`bench.py --calibrate-copy` into HBM bytes per step of the sub-bit convolution kernels.

    python -m paper_2110_09195_amd.hbm_traffic fetch_counter_collection.csv write_counter_collection.csv STEPS

The counters are scaled by what they read for the calibration kernel of bench.py (one elementwise
kernel that reads 256 MiB and writes 256 MiB).  Prints a JSON object (bytes per step, per-kernel
detail and the scale factors); STEPS is the number of bench steps the passes ran (warm-up + timed +
the per-layer timing repetitions all launch the same kernels, so the per-launch average is used).
"""
import collections
import csv
import json
import sys

CAL_BYTES = 64 * 1024 * 1024 * 4


def _per_kernel(path, counter):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            agg[r["Kernel_Name"]].append(float(r["Counter_Value"]) * 1024.0)
    return agg


def _short(name):
    return name.replace("void ", "").replace("snn::(anonymous namespace)::", "").split("(")[0]


def main(fetch_csv, write_csv):
    fetch = _per_kernel(fetch_csv, "FETCH_SIZE")
    write = _per_kernel(write_csv, "WRITE_SIZE")
    cal_f = [v for k, v in fetch.items() if "CUDAFunctorOnSelf_add" in k][0]
    cal_w = [v for k, v in write.items() if "CUDAFunctorOnSelf_add" in k][0]
    sf = CAL_BYTES / (sum(cal_f) / len(cal_f))
    sw = CAL_BYTES / (sum(cal_w) / len(cal_w))
    out = {"unit": "bytes per step (all launches of the sub-bit conv kernels in one step)",
           "fetch_scale": sf, "write_scale": sw, "kernels": {}}
    total_f = total_w = 0.0
    launches_per_step = {}
    for k, v in fetch.items():
        if "subbit_mfma_kernel" in k or "subbit_direct_kernel" in k:
            w = write.get(k, [0.0])
            # launches of this kernel per step: ResNet-18 stack -> count layers by instantiation
            out["kernels"][_short(k)] = {"launches": len(v), "fetch_bytes_per_launch": sf * sum(v) / len(v),
                                         "write_bytes_per_launch": sw * sum(w) / len(w)}
    return out, sf, sw


if __name__ == "__main__":
    res, sf, sw = main(sys.argv[1], sys.argv[2])
    per_step_launches = json.loads(sys.argv[3]) if len(sys.argv) > 3 else None
    if per_step_launches:
        f = sum(res["kernels"][k]["fetch_bytes_per_launch"] * n for k, n in per_step_launches.items())
        w = sum(res["kernels"][k]["write_bytes_per_launch"] * n for k, n in per_step_launches.items())
        res["fetch_bytes"] = f
        res["write_bytes"] = w
        res["bytes"] = f + w
    print(json.dumps(res, indent=1))
