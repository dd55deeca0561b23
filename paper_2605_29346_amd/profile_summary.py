"""Turns a `rocprofv3 --kernel-trace --stats --output-format csv` output folder into the short text
summary kept under profiles/: per-kernel launch statistics of the library's kernels and the GPU-busy
fraction (union of kernel execution intervals / wall time, the paper's "GPU execution fraction")
over the steady-state steps.

    python -m paper_2605_29346_amd.profile_summary <folder> <prefix> [--skip-steps W] [--cmd "..."] > profiles/x.md
"""
from __future__ import annotations

import argparse
import csv
import os
from collections import defaultdict


def short(name: str) -> str:
    name = name.replace("void ", "").replace("zg::", "")
    return name.split("(")[0]


def pmc_main(argv) -> None:
    """pmc <fetch_counter_collection.csv> <write_counter_collection.csv> [--traffic-out file] [--cmd "..."]:
    HBM bytes per launch of the library's kernels from FETCH_SIZE / WRITE_SIZE, each scaled by what the same
    counter reads for the probe's calibration kernel (which reads and writes a known number of bytes)."""
    from .traffic_probe import CALIB_BYTES, CALIB_ELEMS
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_csv")
    ap.add_argument("write_csv")
    ap.add_argument("--traffic-out", default="")
    ap.add_argument("--cmd", default="")
    ap.add_argument("--last", type=int, default=20, help="use the last N launches of each kernel (the timed steps)")
    args = ap.parse_args(argv)

    def load(path, counter):
        per_kernel, calib = defaultdict(list), []
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            name, val = r["Kernel_Name"], float(r["Counter_Value"])
            if "zg::" in name:
                per_kernel[short(name)].append(val)
            elif "MulFunctor<float>" in name and int(r["Grid_Size"]) in (CALIB_ELEMS // 4, CALIB_ELEMS):
                calib.append(val)  # the probe's dst = src * 1 (torch gives each lane 4 elements)
        return per_kernel, calib

    fetch, fcal = load(args.fetch_csv, "FETCH_SIZE")
    write, wcal = load(args.write_csv, "WRITE_SIZE")
    assert fcal and wcal, "calibration kernel not found in the counter files"
    f_unit = CALIB_BYTES / (sum(fcal) / len(fcal))  # bytes per counter unit
    w_unit = CALIB_BYTES / (sum(wcal) / len(wcal))
    print("# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary")
    if args.cmd:
        print(f"\ncommands: {args.cmd}")
    print(f"\ncalibration kernel (dst = src * 1, {CALIB_BYTES} bytes read and {CALIB_BYTES} written): FETCH_SIZE reads "
          f"{sum(fcal) / len(fcal):.1f}, WRITE_SIZE reads {sum(wcal) / len(wcal):.1f} -> {f_unit:.1f} and {w_unit:.1f} bytes per unit "
          f"(1 KiB = 1024)")
    print("\n| kernel | launches used | FETCH_SIZE avg | WRITE_SIZE avg | HBM read MB | HBM write MB |")
    print("|---|---|---|---|---|---|")
    lines = []
    for k in sorted(fetch):
        f = fetch[k][-args.last:]
        w = write.get(k, [0.0])[-args.last:]
        fb, wb = f_unit * sum(f) / len(f), w_unit * sum(w) / len(w)
        print(f"| {k} | {len(f)} | {sum(f) / len(f):.1f} | {sum(w) / len(w):.1f} | {fb / 1e6:.2f} | {wb / 1e6:.2f} |")
        lines.append(f"{k.split('<')[0]} {fb:.0f} {wb:.0f}")
    if args.traffic_out:
        with open(args.traffic_out, "w") as fh:
            fh.write("# kernel  hbm_read_bytes_per_launch  hbm_write_bytes_per_launch  (from the summary beside this file)\n")
            fh.write("\n".join(lines) + "\n")


def hipapi_main(argv) -> None:
    """hipapi <hip_api_trace.csv> [--warmup W] [--cmd "..."]: the HIP API calls the host makes between the first
    and the last timed step of bench.py (every step is one hipGraphLaunch): shows that the steady-state loop
    contains no synchronising call, no copy and no allocation."""
    ap = argparse.ArgumentParser()
    ap.add_argument("trace_csv")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--cmd", default="")
    args = ap.parse_args(argv)
    rows = sorted(csv.DictReader(open(args.trace_csv)), key=lambda r: int(r["Start_Timestamp"]))
    launches = [i for i, r in enumerate(rows) if r["Function"] == "hipGraphLaunch"]
    print("# rocprofv3 --hip-trace summary: host API calls inside the timed loop")
    if args.cmd:
        print(f"\ncommand: `{args.cmd}`")
    print(f"\nhipGraphLaunch calls in the run: {len(launches)} ({args.warmup} warm-up steps left out below)")
    a, b = launches[args.warmup], launches[-1]
    inside = defaultdict(int)
    for r in rows[a:b + 1]:
        inside[r["Function"]] += 1
    print("\n| HIP API call between the first and the last timed launch | calls |")
    print("|---|---|")
    for k, v in sorted(inside.items(), key=lambda kv: -kv[1]):
        print(f"| {k} | {v} |")
    sync = [k for k in inside if "Synchronize" in k or "Memcpy" in k or "Malloc" in k or k.startswith("hipEventQuery")]
    print(f"\nsynchronising / copying / allocating calls inside the loop: {sync if sync else 'none'}")
    print(f"first call after the loop: {rows[b + 1]['Function'] if b + 1 < len(rows) else '-'} ... "
          f"{next((r['Function'] for r in rows[b + 1:] if 'Synchronize' in r['Function']), '-')} (the one sync that ends the timed region)")


def main() -> None:
    import sys
    if len(sys.argv) > 1 and sys.argv[1] == "pmc":
        pmc_main(sys.argv[2:])
        return
    if len(sys.argv) > 1 and sys.argv[1] == "hipapi":
        hipapi_main(sys.argv[2:])
        return
    ap = argparse.ArgumentParser()
    ap.add_argument("folder")
    ap.add_argument("prefix")
    ap.add_argument("--skip-steps", type=int, default=10, help="warm-up steps to leave out of the busy fraction")
    ap.add_argument("--cmd", default="")
    ap.add_argument("--window-only", action="store_true", help="per-kernel durations over the counted steps only")
    ap.add_argument("--note", default="")
    args = ap.parse_args()
    trace = list(csv.DictReader(open(os.path.join(args.folder, f"{args.prefix}_kernel_trace.csv"))))
    ours = [r for r in trace if "zg::" in r["Kernel_Name"]]
    ours.sort(key=lambda r: int(r["Start_Timestamp"]))
    ingest = [i for i, r in enumerate(ours) if "k_ingest" in r["Kernel_Name"]]
    print("# rocprofv3 kernel-trace summary")
    if args.cmd:
        print(f"\ncommand: `{args.cmd}`")
    if args.note:
        print(f"\n{args.note}")
    print(f"\nkernel dispatches of the library: {len(ours)}; steps (ingest kernels): {len(ingest)}")

    seg = None
    if len(ingest) > args.skip_steps + 1:
        first = ingest[args.skip_steps]
        # steady-state window: from the first counted step's ingest to the end of the last step (stand-alone
        # kernel launches after the last step are not part of the loop)
        last = ingest[-1]
        per_step = -(-(ingest[-1] - first) // (len(ingest) - 1 - args.skip_steps))
        seg = ours[first: last + per_step]

    stats = defaultdict(list)
    for r in (seg if (args.window_only and seg) else ours):
        stats[short(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    total = sum(sum(v) for v in stats.values())
    where = f"the {len(ingest) - args.skip_steps} steps after the first {args.skip_steps}" if (args.window_only and seg) else "the whole run"
    print(f"\nper-kernel durations over {where}:")
    print("\n| kernel | launches | avg us | min us | max us | share of library GPU time |")
    print("|---|---|---|---|---|---|")
    for k, v in sorted(stats.items(), key=lambda kv: -sum(kv[1])):
        print(f"| {k} | {len(v)} | {sum(v) / len(v) / 1e3:.2f} | {min(v) / 1e3:.2f} | {max(v) / 1e3:.2f} | {100 * sum(v) / total:.1f}% |")

    if seg:
        t0 = int(seg[0]["Start_Timestamp"])
        t1 = max(int(r["End_Timestamp"]) for r in seg)
        ivs = sorted((int(r["Start_Timestamp"]), int(r["End_Timestamp"])) for r in seg)
        busy, cur_s, cur_e = 0, ivs[0][0], ivs[0][1]
        for s, e in ivs[1:]:
            if s > cur_e:
                busy += cur_e - cur_s
                cur_s, cur_e = s, e
            else:
                cur_e = max(cur_e, e)
        busy += cur_e - cur_s
        nsteps = len(ingest) - args.skip_steps
        print(f"\nsteady state: {nsteps} steps, about {per_step} kernels per step, wall {1e-3 * (t1 - t0):.1f} us "
              f"({1e-3 * (t1 - t0) / nsteps:.2f} us/step), union of kernel intervals {1e-3 * busy:.1f} us")
        print(f"\n**GPU-busy fraction = {100.0 * busy / (t1 - t0):.2f}%**")


if __name__ == "__main__":
    main()
