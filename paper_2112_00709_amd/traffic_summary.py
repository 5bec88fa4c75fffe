"""HBM traffic of the LF-MMI call's kernels from two rocprofv3 counter runs.

Usage (on the GPU machine, from the repository root; one counter per run):

    export FB_AMD_SERIAL=1
    rocprofv3 --pmc FETCH_SIZE -d out/pmc_fetch -o p --output-format csv -- \\
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-context --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d out/pmc_write -o p --output-format csv -- \\
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-context --calibrate-copy
    python3 -m paper_2112_00709_amd.traffic_summary out/pmc_fetch out/pmc_write \\
        profiles/lfmmi_config5_traffic.json

FB_AMD_SERIAL=1 keeps every launch of a call on the caller's stream.  A counter run lets one kernel at a time onto
the GPU, and the LF-MMI call's stream waits on progress words are small spinning kernels: one that is let on before
the launch it waits for would never end.  The kernels and their traffic are the same either way.

Both counters are in KiB per dispatch.  They are scaled by what the same counter reads for the plain device copies
of the run (`bench.py` copies 1 GiB several times: 1 GiB read and 1 GiB written per copy are the true figures), and
summed per kernel and per LF-MMI call.  The output names the kernel whose figures `bench.py` reports as
`roofline.traffic`, so that a renamed or replaced kernel shows as a missing figure instead of a stale one.
"""
from __future__ import annotations

import csv
import glob
import json
import os
import subprocess
import sys

COPY_KERNEL = "copyBuffer"          # the runtime's device-to-device copy kernel
COPY_BYTES = 1 << 30                # bench.py copies 2^28 floats
DOMINANT = "fb_linear_kernel"
LOSS = "fb_loss_kernel"             # once per LF-MMI call
COPY_MIN_KIB = 100 * 1024           # the run also holds small copies: only the big ones calibrate


def read_counter(folder: str, counter: str):
    """kernel name -> (dispatches, sum of the counter over them); of the copy kernel only the 1 GiB copies."""
    paths = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
    if not paths:
        raise SystemExit(f"no *counter_collection.csv under {folder}")
    per_dispatch = {}
    for path in paths:
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] != counter:
                    continue
                key = (path, row["Dispatch_Id"], row["Kernel_Name"])
                per_dispatch[key] = per_dispatch.get(key, 0.0) + float(row["Counter_Value"])
    out = {}
    for (_, _, name), kib in per_dispatch.items():
        if COPY_KERNEL in name and kib < COPY_MIN_KIB:
            continue
        n, tot = out.get(name, (0, 0.0))
        out[name] = (n + 1, tot + kib)
    return out


def short(name: str) -> str:
    head = name.split("(")[0]
    return head.replace("void ", "").replace("fb::", "")


def main(argv) -> int:
    if len(argv) != 4:
        print(__doc__, file=sys.stderr)
        return 2
    fetch, write = read_counter(argv[1], "FETCH_SIZE"), read_counter(argv[2], "WRITE_SIZE")

    def total(tab, needle):
        n = sum(v[0] for k, v in tab.items() if needle in k)
        kib = sum(v[1] for k, v in tab.items() if needle in k)
        return n, kib

    n_copy_f, copy_f = total(fetch, COPY_KERNEL)
    n_copy_w, copy_w = total(write, COPY_KERNEL)
    if not n_copy_f or not n_copy_w or copy_f <= 0 or copy_w <= 0:
        raise SystemExit("no plain copies in the runs: pass --calibrate-copy to bench.py")
    scale_f = n_copy_f * COPY_BYTES / (copy_f * 1024.0)
    scale_w = n_copy_w * COPY_BYTES / (copy_w * 1024.0)
    calls_f, calls_w = total(fetch, LOSS)[0], total(write, LOSS)[0]
    if not calls_f or calls_f != calls_w:
        raise SystemExit("the two runs hold different numbers of LF-MMI calls")
    kernels = {}
    for name in sorted(set(fetch) | set(write)):
        if "fb::" not in name:
            continue
        nf, kf = fetch.get(name, (0, 0.0))
        nw, kw = write.get(name, (0, 0.0))
        kernels[short(name)] = {
            "dispatches_per_call": nf / calls_f,
            "fetch_kib_per_call": kf / calls_f, "write_kib_per_call": kw / calls_w,
            "traffic_bytes_per_call": (kf / calls_f * scale_f + kw / calls_w * scale_w) * 1024.0}
    dom = [k for k in kernels if DOMINANT in k]
    if len(dom) != 1:
        raise SystemExit(f"expected one kernel named {DOMINANT}, found {dom}")
    d = kernels[dom[0]]
    try:
        git = subprocess.run(["git", "rev-parse", "HEAD"], stdout=subprocess.PIPE, text=True, check=True,
                             cwd=os.path.dirname(os.path.abspath(__file__))).stdout.strip()
    except (OSError, subprocess.CalledProcessError):
        git = None
    result = {
        "workload": "config5, lfmmi_loss_grad",
        "kernel": dom[0],
        "launches_per_call": d["dispatches_per_call"],
        "fetch_kib_per_launch": d["fetch_kib_per_call"] / d["dispatches_per_call"],
        "write_kib_per_launch": d["write_kib_per_call"] / d["dispatches_per_call"],
        "fetch_scale": scale_f, "write_scale": scale_w,
        "traffic_bytes_per_launch": d["traffic_bytes_per_call"] / d["dispatches_per_call"],
        "whole_call_traffic_bytes": sum(k["traffic_bytes_per_call"] for k in kernels.values()),
        "calls": calls_f, "copies": n_copy_f, "kernels": kernels, "git": git,
    }
    with open(argv[3], "w") as f:
        json.dump(result, f, indent=1)
        f.write("\n")
    print(json.dumps({k: result[k] for k in ("kernel", "traffic_bytes_per_launch", "whole_call_traffic_bytes",
                                             "fetch_scale", "write_scale", "calls")}))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
