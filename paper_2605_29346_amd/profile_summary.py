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


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("folder")
    ap.add_argument("prefix")
    ap.add_argument("--skip-steps", type=int, default=10, help="warm-up steps to leave out of the busy fraction")
    ap.add_argument("--cmd", default="")
    args = ap.parse_args()
    trace = list(csv.DictReader(open(os.path.join(args.folder, f"{args.prefix}_kernel_trace.csv"))))
    ours = [r for r in trace if "zg::" in r["Kernel_Name"]]
    ours.sort(key=lambda r: int(r["Start_Timestamp"]))
    ingest = [i for i, r in enumerate(ours) if "k_ingest" in r["Kernel_Name"]]
    print("# rocprofv3 kernel-trace summary")
    if args.cmd:
        print(f"\ncommand: `{args.cmd}`")
    print(f"\nkernel dispatches of the library: {len(ours)}; steps (ingest kernels): {len(ingest)}")

    stats = defaultdict(list)
    for r in ours:
        stats[short(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    total = sum(sum(v) for v in stats.values())
    print("\n| kernel | launches | avg us | min us | max us | share of library GPU time |")
    print("|---|---|---|---|---|---|")
    for k, v in sorted(stats.items(), key=lambda kv: -sum(kv[1])):
        print(f"| {k} | {len(v)} | {sum(v) / len(v) / 1e3:.2f} | {min(v) / 1e3:.2f} | {max(v) / 1e3:.2f} | {100 * sum(v) / total:.1f}% |")

    if len(ingest) > args.skip_steps + 1:
        first = ingest[args.skip_steps]
        # steady-state window: from the first timed step's ingest to the last step-ending kernel
        step_end = max(i for i, r in enumerate(ours) if any(t in r["Kernel_Name"] for t in ("k_finish", "k_tail", "k_aggregate")) and i >= ingest[-1])
        # stand-alone kernel launches after the last step are not part of the loop: stop at the first
        # kernel that follows the last ingest's step
        last = ingest[-1]
        per_step = (ingest[-1] - first) // (len(ingest) - 1 - args.skip_steps)
        seg = ours[first: last + per_step]
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
        print(f"\nsteady state: {nsteps} steps, {per_step} kernels per step, wall {1e-3 * (t1 - t0):.1f} us "
              f"({1e-3 * (t1 - t0) / nsteps:.2f} us/step), union of kernel intervals {1e-3 * busy:.1f} us")
        print(f"\n**GPU-busy fraction = {100.0 * busy / (t1 - t0):.2f}%**")


if __name__ == "__main__":
    main()
