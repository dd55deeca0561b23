#!/usr/bin/env python3
"""Throughput of the whole mini-batch construction step on one MI355X.

One "step" = one pass of the hot path (sample -> dedup/relabel -> block CSR -> gather -> mean
aggregation) over one synthetic mini-batch, issued through the C-ABI library as one ingest kernel
plus one hipGraph replay, with no host synchronisation between steps.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload very_large] [--env model|max|graph] [--extras]

The default workload is the largest single-GPU configuration (110 M vertices, 1.5 B edges, 56 GB of
features resident in HBM).  Besides the headline value the line carries
  roofline     - the dominant kernel of the step (gather or aggregate): algorithmic bytes per launch
                 / its average launch duration, measured here with events on the launch stream,
                 against MI355X's 8 TB/s HBM peak;
  cpu_baseline - the CPU checker (oracle/, untuned) timed on this machine's host cores on a bounded
                 sample of the same steps.

Two more modes serve the profiles kept under profiles/ (every command recorded there runs this file only):
    python bench.py --profile-loop [--workload W] [--pipeline P] [--steps K]
        a short steady-state loop plus three launches of the library's calibration copy, and nothing else: the
        program to put behind `rocprofv3 --kernel-trace --stats`, `--hip-trace` or `--pmc FETCH_SIZE|WRITE_SIZE`
    python bench.py --summarize kernel <folder> <prefix> [--skip-steps W] [--window-only] [--cmd ...] [--note ...]
    python bench.py --summarize pmc <fetch_counter_collection.csv> <write_counter_collection.csv> [--traffic-out f] [--cmd ...]
    python bench.py --summarize hipapi <hip_api_trace.csv> [--warmup W] [--cmd ...]
        turn rocprofv3's csv output into the short text summaries (no GPU needed)
"""
import argparse
import csv
import json
import os
import sys
import time
from collections import defaultdict
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


CALIB_BYTES = (96 * 1024 * 1024 + 4096) * 4  # the calibration copy reads and writes this many bytes


def read_traffic_summary(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, if there is one
    (profiles/hbm_traffic_<workload>.txt, lines `<kernel> <fetch_bytes> <write_bytes>`) AND it was taken from the
    kernels as they are now: the file names the hash of the library's sources it was measured on, and a summary
    of other sources is not reported (None)."""
    from paper_2605_29346_amd import build as zg_build
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    lines = open(path).read().splitlines()
    if not any(l.startswith("# sources ") and l.split()[2] == zg_build.source_id() for l in lines):
        return None
    for line in lines:
        parts = line.split()
        if len(parts) >= 3 and parts[0] == kernel:
            try:
                return float(parts[1]) + float(parts[2])
            except ValueError:
                return None
    return None


# --------------------------------------------------------------------------------------------------
# summaries of rocprofv3 csv output (no GPU needed)
# --------------------------------------------------------------------------------------------------
def _short(name: str) -> str:
    return name.replace("void ", "").replace("zg::", "").split("(")[0]


def summarize_pmc(argv) -> None:
    """HBM bytes per launch of the library's kernels from FETCH_SIZE / WRITE_SIZE, each scaled by what the same
    counter reads for the library's calibration copy (which reads and writes a known number of bytes)."""
    from paper_2605_29346_amd import build as zg_build
    ap = argparse.ArgumentParser(prog="bench.py --summarize pmc")
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
            if "k_calibrate_copy" in name:
                calib.append(val)
            elif "zg::" in name:
                label = _short(name)
                if "k_hop" in label and r.get("Grid_Size") and r.get("Workgroup_Size"):  # a step's hop launches, told apart by grid
                    label += f"[{int(r['Grid_Size']) // int(r['Workgroup_Size'])}wg]"
                per_kernel[label].append(val)
        return per_kernel, calib

    fetch, fcal = load(args.fetch_csv, "FETCH_SIZE")
    write, wcal = load(args.write_csv, "WRITE_SIZE")
    assert fcal and wcal, "calibration kernel not found in the counter files"
    f_unit = CALIB_BYTES / (sum(fcal) / len(fcal))  # bytes per counter unit
    w_unit = CALIB_BYTES / (sum(wcal) / len(wcal))
    print("# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary")
    if args.cmd:
        print(f"\ncommands: {args.cmd}")
    print(f"\ncalibration kernel (the library's plain copy, {CALIB_BYTES} bytes read and {CALIB_BYTES} written): FETCH_SIZE reads "
          f"{sum(fcal) / len(fcal):.1f}, WRITE_SIZE reads {sum(wcal) / len(wcal):.1f} -> {f_unit:.1f} and {w_unit:.1f} bytes per unit "
          f"(1 KiB = 1024)")
    print(f"\nlibrary sources: {zg_build.source_id()}")
    print("\n| kernel | launches used | FETCH_SIZE avg | WRITE_SIZE avg | HBM read MB | HBM write MB |")
    print("|---|---|---|---|---|---|")
    lines = []
    for k in sorted(fetch):
        f = fetch[k][-args.last:]
        w = write.get(k, [0.0])[-args.last:]
        fb, wb = f_unit * sum(f) / len(f), w_unit * sum(w) / len(w)
        print(f"| {k} | {len(f)} | {sum(f) / len(f):.1f} | {sum(w) / len(w):.1f} | {fb / 1e6:.2f} | {wb / 1e6:.2f} |")
        lines.append(f"{k.split('<')[0] + (k[k.index('['):] if '[' in k else '')} {fb:.0f} {wb:.0f}")
    if args.traffic_out:
        with open(args.traffic_out, "w") as fh:
            fh.write("# kernel  hbm_read_bytes_per_launch  hbm_write_bytes_per_launch  (from the summary beside this file)\n")
            fh.write(f"# sources {zg_build.source_id()}\n")
            fh.write("\n".join(lines) + "\n")


def summarize_hipapi(argv) -> None:
    """The HIP API calls the host makes between the first and the last timed step (every step is one
    hipGraphLaunch): shows that the steady-state loop holds no synchronising call, no copy and no allocation."""
    ap = argparse.ArgumentParser(prog="bench.py --summarize hipapi")
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


def summarize_kernel(argv) -> None:
    """Per-kernel launch statistics of the library's kernels and the GPU-busy fraction (union of kernel execution
    intervals / wall time, the paper's "GPU execution fraction") over the steady-state steps."""
    ap = argparse.ArgumentParser(prog="bench.py --summarize kernel")
    ap.add_argument("folder")
    ap.add_argument("prefix")
    ap.add_argument("--skip-steps", type=int, default=10, help="warm-up steps to leave out of the busy fraction")
    ap.add_argument("--cmd", default="")
    ap.add_argument("--window-only", action="store_true", help="per-kernel durations over the counted steps only")
    ap.add_argument("--note", default="")
    args = ap.parse_args(argv)
    trace = list(csv.DictReader(open(os.path.join(args.folder, f"{args.prefix}_kernel_trace.csv"))))
    ours = [r for r in trace if "zg::" in r["Kernel_Name"] and "k_calibrate_copy" not in r["Kernel_Name"]]
    ours.sort(key=lambda r: int(r["Start_Timestamp"]))
    # every step ends with one k_aggregate launch (its last workgroups close the step); the profiled loop holds nothing else
    steps = sum(1 for r in ours if "k_aggregate" in r["Kernel_Name"])
    print("# rocprofv3 kernel-trace summary")
    if args.cmd:
        print(f"\ncommand: `{args.cmd}`")
    if args.note:
        print(f"\n{args.note}")
    print(f"\nkernel dispatches of the library: {len(ours)}; steps: {steps}")

    seg = None
    per_step = len(ours) // steps if steps else 0
    if steps > args.skip_steps + 1 and per_step * steps == len(ours):
        # steady-state window: the dispatches after the warm-up steps' share (with several plans in flight the steps
        # interleave, so the cut is by dispatch count, in start order)
        seg = ours[args.skip_steps * per_step:]
    ingest = list(range(steps))

    def label(r):
        # the hop kernel's launches of a step share a name: tell them apart by their grid (workgroups of 1024 lanes)
        name = _short(r["Kernel_Name"])
        if "k_hop" in name and r.get("Grid_Size_X") and r.get("Workgroup_Size_X"):
            name += f" [{int(r['Grid_Size_X']) // int(r['Workgroup_Size_X'])} workgroups]"
        return name

    stats = defaultdict(list)
    for r in (seg if (args.window_only and seg) else ours):
        stats[label(r)].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
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


# --------------------------------------------------------------------------------------------------
# the benchmark
# --------------------------------------------------------------------------------------------------
def main():
    if len(sys.argv) > 2 and sys.argv[1] == "--summarize":
        {"kernel": summarize_kernel, "pmc": summarize_pmc, "hipapi": summarize_hipapi}[sys.argv[2]](sys.argv[3:])
        return
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="very_large",
                    help="tiny | medium_dense | large_sparse | very_large (default: the largest single-GPU configuration) | envelope_stress")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only; invalid as a result)")
    ap.add_argument("--env", default="model", choices=["model", "max", "graph"],
                    help="envelope of the plans: the paper's Lemma 1 from the degree histogram (default), the worst case, or "
                         "the lemma's cap formula on the graph-aware size model")
    ap.add_argument("--eager", action="store_true", help="plans launch their kernels one by one instead of replaying a hipGraph "
                    "(a comparison; the default and the reported configuration is the captured graph)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--extras", action="store_true", help="also time the ZG_PLAN_FUSED_INPUT and ZG_PLAN_AUTO_FALLBACK plan "
                    "variants and report the graph-aware envelope (extra keys; the headline is unchanged)")
    ap.add_argument("--pipeline", type=int, default=4,
                    help="independent plans replayed round-robin on their own streams (consecutive mini-batches do not "
                         "depend on each other); 1 = strictly one step after the other")
    ap.add_argument("--input-cache", default="", help="folder for the generated graph and seed batches (.npy): written when "
                    "absent, loaded otherwise, so that a profiled run launches none of the generator's kernels")
    ap.add_argument("--empty-features", action="store_true", help="--profile-loop only: leave the feature table uninitialised "
                    "(memory traffic and timing do not depend on the values; results are not checked in this mode)")
    ap.add_argument("--profile-loop", action="store_true", help="only the steady-state loop (on --pipeline plans) and three "
                    "launches of the calibration copy: the program to run under rocprofv3")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a single-GPU path (no sharding, no collectives); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2605_29346_amd import workloads as W
    from paper_2605_29346_amd import zg

    zg.lib()  # loads what is built (rebuilt only if missing or stale); fails loudly if there is no library: no other path
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"

    cfg = W.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = cfg.scaled(args.scale)
    K, Wm = args.steps, args.warmup

    t0 = time.time()
    cache = os.path.join(args.input_cache, f"{cfg.name}_{K + Wm}") if args.input_cache else ""
    pool = None
    if cache and os.path.exists(cache + "_batches.npy"):
        g = W.Graph(0, torch.from_numpy(np.load(cache + "_offsets.npy")).to(dev), torch.from_numpy(np.load(cache + "_indices.npy")).to(dev))
        g.num_nodes = g.offsets.numel() - 1
        batches = list(torch.from_numpy(np.load(cache + "_batches.npy")).to(dev))
        log(f"[bench] graph {cfg.name} and {len(batches)} seed batches loaded from {args.input_cache} ({time.time() - t0:.1f}s)")
    else:
        g = cfg.build_graph(device=dev)
        pool = cfg.seed_pool(g)
        batches = [pool.batch_for(s).contiguous() for s in range(K + Wm)]
        torch.cuda.synchronize()
        log(f"[bench] graph {cfg.name}: |V|={g.num_nodes} |E|={g.num_edges}, {len(batches)} seed batches ({time.time() - t0:.1f}s)")
        if cache:
            os.makedirs(args.input_cache, exist_ok=True)
            np.save(cache + "_offsets.npy", g.offsets.cpu().numpy())
            np.save(cache + "_indices.npy", g.indices.cpu().numpy())
            np.save(cache + "_batches.npy", torch.stack(batches).cpu().numpy())
            log(f"[bench] inputs written to {args.input_cache} ({time.time() - t0:.1f}s)")
    keys = [cfg.key_for(s) for s in range(K + Wm)]
    t0 = time.time()
    if args.empty_features and args.profile_loop:
        feat = torch.empty((g.num_nodes, cfg.dim), dtype=torch.float32, device=dev)
    else:
        feat = W.feature_table(g.num_nodes, cfg.dim, cfg.feat_seed, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] features {tuple(feat.shape)} ({time.time() - t0:.1f}s)")

    dg = zg.Graph(g.offsets, g.indices)
    H = len(cfg.fanouts)

    def make_plan(mode, flags=0):
        flags |= zg.PLAN_EAGER if args.eager else 0
        if mode == "graph":
            assert pool is not None, "--env graph needs the seed pool: do not combine it with a loaded --input-cache"
            env = zg.graph_envelope(dg, cfg.fanouts, cfg.batch, flags=flags, seed_prob=pool.seed_prob(g.num_nodes))
        else:
            env = zg.make_envelope(zg.ENV_MODEL if mode == "model" else zg.ENV_MAX, flags=flags)
        p = zg.Plan(dg, cfg.fanouts, cfg.batch, env, feat_dim=cfg.dim)
        p.bind_features(feat)
        return p

    def run(plans, streams):
        P = len(plans)
        for s in range(Wm):
            plans[s % P].step(batches[s], keys[s], streams[s % P])
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for s in range(Wm, Wm + K):
            plans[s % P].step(batches[s], keys[s], streams[s % P])
        t_issued = time.perf_counter() - t_start
        torch.cuda.synchronize()
        t_all = time.perf_counter() - t_start
        log(f"[bench] {P} stream(s): host issued {K} steps in {t_issued * 1e3:.2f} ms, device finished after {t_all * 1e3:.2f} ms")
        return t_all

    def flags_of(plans):
        f = 0
        for p in plans:
            f |= int(p.view_counts()[3].cpu()[0]) & 0xFFFFFFFF
        return f

    cur = torch.cuda.current_stream()
    if args.profile_loop:
        P = max(1, args.pipeline)
        plans = [make_plan(args.env) for _ in range(P)]
        streams = [cur] if P == 1 else [zg.new_stream() for _ in plans]
        torch.cuda.synchronize()
        wall = run(plans, streams)
        assert flags_of(plans) == 0, f"device status flags {flags_of(plans):#x}"
        src = torch.ones(CALIB_BYTES // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            zg.calibration_copy(src, dst)
        torch.cuda.synchronize()
        n, E, _, _ = [t.cpu().tolist() for t in plans[0].view_counts()]
        log(f"[bench] profile loop: {cfg.name}, {P} plan(s), {K} steps in {wall * 1e3:.2f} ms ({wall / K * 1e6:.1f} us/step); "
            f"last step n={n} E={E}; calibration copy of {CALIB_BYTES} bytes x3")
        return

    env_mode = args.env
    plan = make_plan(env_mode)
    wall_single = run([plan], [cur])
    if flags_of([plan]) and env_mode != "max":
        log(f"[bench] the {env_mode} envelope overflowed (flags {flags_of([plan]):#x}); re-running on the worst-case envelope")
        env_mode = "max"
        plan = make_plan(env_mode)
        wall_single = run([plan], [cur])
    assert flags_of([plan]) == 0, f"device status flags {flags_of([plan]):#x}"
    wall, pipeline = wall_single, 1
    if args.pipeline > 1:
        plans = [plan] + [make_plan(env_mode) for _ in range(args.pipeline - 1)]
        streams = [zg.new_stream() for _ in plans]  # own streams: they map to distinct hardware queues
        torch.cuda.synchronize()
        wall_pipe = run(plans, streams)
        assert flags_of(plans) == 0, f"device status flags {flags_of(plans):#x}"
        log(f"[bench] one stream: {K / wall_single:.0f} steps/s; {args.pipeline} plans on {args.pipeline} streams: {K / wall_pipe:.0f} steps/s")
        if wall_pipe < wall_single:
            wall, pipeline = wall_pipe, args.pipeline
        # the size log below is read from the first plan: replay the timed steps' sizes on it alone
        plan = plans[0]
    ms_per_step = wall / K * 1e3
    value = K / wall

    fused = auto_fb = gm = None
    if args.extras:
        # extra (not the headline): the same steps with plans that materialise only the frontier's rows of X and
        # aggregate straight from the feature table (what the first GraphSAGE layer needs)
        fplans = [make_plan(env_mode, zg.PLAN_FUSED_INPUT) for _ in range(max(1, args.pipeline))]
        fstreams = [zg.new_stream() for _ in fplans]
        torch.cuda.synchronize()
        wf1 = run(fplans[:1], [cur])
        wfp = run(fplans, fstreams) if len(fplans) > 1 else wf1
        assert flags_of(fplans) == 0
        fused = {"value": K / min(wf1, wfp), "single_stream_value": K / wf1, "envelope_bytes": int(fplans[0].info.envelope_bytes),
                 "note": "ZG_PLAN_FUSED_INPUT: X holds the rows of D_{H-1} only, the mean reads its input rows from the table"}
        log(f"[bench] fused input: one stream {K / wf1:.0f} steps/s; pipelined {K / wfp:.0f} steps/s")
        for fp in fplans:
            fp.close()
        del fplans

        # extra: what the device-side fallback conditional costs when it never fires (the twin's gated kernels
        # return at once; the plan itself is the same model envelope)
        if env_mode != "max":
            aplans = [make_plan(env_mode, zg.PLAN_AUTO_FALLBACK) for _ in range(max(1, args.pipeline))]
            astreams = [zg.new_stream() for _ in aplans]
            torch.cuda.synchronize()
            wa1 = run(aplans[:1], [cur])
            wap = run(aplans, astreams) if len(aplans) > 1 else wa1
            fell = sum(int(p.safe_view().epoch()) for p in aplans)
            auto_fb = {"value": K / min(wa1, wap), "single_stream_value": K / wa1, "fallbacks": fell,
                       "safe_envelope_bytes": int(aplans[0].info.safe_envelope_bytes),
                       "note": "ZG_PLAN_AUTO_FALLBACK: the worst-case twin's kernels ride in every step's graph behind a device-side gate"}
            log(f"[bench] automatic fallback armed: one stream {K / wa1:.0f} steps/s; pipelined {K / wap:.0f} steps/s; fell back {fell} times")
            for ap_ in aplans:
                ap_.close()
            del aplans

        # extra: the envelope the graph-aware size model would provision (caps from the inclusion probabilities propagated
        # over the graph itself instead of the lemma's degree-proportional draws), checked against the realised sizes below
        t_gm = time.perf_counter()
        genv = zg.graph_envelope(dg, cfg.fanouts, cfg.batch, seed_prob=pool.seed_prob(g.num_nodes))
        torch.cuda.synchronize()
        t_gm = time.perf_counter() - t_gm
        gm = (dg.plan_query(cfg.fanouts, cfg.batch, genv, feat_dim=cfg.dim), t_gm)

    # realised sizes of the timed steps from the device-side log
    logrec = plan.view_log().cpu().numpy().astype(np.int64)
    total_steps = plan.epoch()
    nrec = min(K, total_steps, logrec.shape[0])
    recs = np.stack([logrec[e % logrec.shape[0]] for e in range(total_steps - nrec, total_steps)])
    n_steps = recs[:, 2:2 + H + 1]
    E_steps = recs[:, 2 + H + 1:2 + 2 * H + 1]
    info = plan.info
    ldx = plan.out.ldx

    def exact_bytes(n, E):
        b = n[H] * 4 + sum((n[h] + 1) * 4 + 2 * E[h] * 4 for h in range(H))
        return b + n[H] * ldx * 4 + n[H - 1] * ldx * 4
    exact = np.array([exact_bytes(n_steps[i], E_steps[i]) for i in range(nrec)], dtype=np.float64)

    # ---- dominant-kernel roofline: stand-alone launches of the very kernels of the step, on the last step's state
    nH, nHm1, EHm1 = int(n_steps[-1][H]), int(n_steps[-1][H - 1]), int(E_steps[-1][H - 1])
    stream = torch.cuda.current_stream()

    def time_kernel(fn):
        # average launch duration: `kernel_reps` launches back to back between one pair of events on the
        # launch stream (so the events' own cost is spread over the launches), best of 3 such runs
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(args.kernel_reps):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            t = a.elapsed_time(b) * 1e-3 / args.kernel_reps
            best = t if best is None else min(best, t)
        return best

    # the step's own two feature launches, replayed on the last step's state: the gather copies the frontier's rows, the
    # aggregation reads its input rows from the table and writes the other rows of X (those of the last hop's new vertices)
    t_gather = time_kernel(lambda: plan.replay_features(0))
    t_agg_replay = time_kernel(lambda: plan.replay_features(1))
    one_pass = bool(plan.out.x_one_pass)
    row = 4 * cfg.dim

    def aggregate_bytes():
        """(compulsory bytes, bytes if every edge fetches its row) of the aggregation launch of the step just run."""
        n_t, E_t, _, _ = plan.view_counts()
        nH_, nHm1_, EHm1_ = int(n_t[H]), int(n_t[H - 1]), int(E_t[H - 1])
        if one_pass:
            # the aggregation reads every distinct row its edges point to at least once (counted exactly, from the
            # step's block), writes the new vertices' rows into X, and writes the means
            distinct = int(torch.unique(plan.view_block(H - 1)[1][:EHm1_]).numel())
            csr = EHm1_ * (4 + 4 + 1) + (nHm1_ + 1) * 4  # sampled ids, local ids (written here), first-edge flags, row_ptr
            return distinct * row + (nH_ - nHm1_) * row + nHm1_ * row + csr, EHm1_ * row + (nH_ - nHm1_) * row + nHm1_ * row + csr
        # two passes: the aggregation reads every row of X at least once and writes the means
        csr = EHm1_ * 4 + (nHm1_ + 1) * 4
        return nH_ * row + nHm1_ * row + csr, EHm1_ * row + nHm1_ * row + csr

    # The aggregation inside real steps: timed steps again on one stream, their kernels enqueued one by one with a pair of
    # events around the aggregation launch (zg_step_timed); duration and bytes of every such launch, averaged per launch.
    probes = min(K, args.kernel_reps)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(probes)]
    for a, b in ev:  # (a first record creates the events' handles)
        a.record(stream)
        b.record(stream)
    torch.cuda.synchronize()
    sum_t = sum_b = sum_bn = 0.0
    for i, (a, b) in enumerate(ev):
        # an ordinary step first, without a sync: while the device works on it the host has the timed step's launches
        # enqueued, as in the steady-state loop (alone, a short step's aggregation would wait for the host's next call)
        plan.step(batches[Wm + (i - 1) % K], keys[Wm + (i - 1) % K])
        plan.step_timed(batches[Wm + i], keys[Wm + i], a, b)
        torch.cuda.synchronize()
        sum_t += a.elapsed_time(b) * 1e-3
        ba, bn = aggregate_bytes()
        sum_b += ba
        sum_bn += bn
    t_agg, bytes_agg, bytes_agg_noreuse = sum_t / probes, int(round(sum_b / probes)), int(round(sum_bn / probes))
    n_new = nH - nHm1
    gather_rows = nHm1 if one_pass else nH
    bytes_gather = gather_rows * (4 + 2 * row)
    kernels = {
        "gather": {"seconds": t_gather, "bytes": bytes_gather, "GBps": bytes_gather / t_gather / 1e9,
                   "name": "k_gather", "rows": gather_rows},
        # `bytes` is the compulsory figure; without cache reuse every edge fetches its row
        "aggregate": {"seconds": t_agg, "bytes": bytes_agg, "GBps": bytes_agg / t_agg / 1e9, "name": "k_aggregate",
                      "bytes_without_reuse": bytes_agg_noreuse, "GBps_without_reuse": bytes_agg_noreuse / t_agg / 1e9,
                      "rows_read_per_edge": EHm1, "x_rows_written": n_new if one_pass else 0,
                      "measured": f"inside {probes} of the timed steps (zg_step_timed: events around the launch), averaged per launch",
                      "seconds_replayed_back_to_back": t_agg_replay},
    }
    dom = max(kernels, key=lambda k: kernels[k]["seconds"])
    roofline = {"bound": "hbm", "kernel": kernels[dom]["name"], "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kernels[dom]["GBps"] / HBM_PEAK_GBS,
                "traffic": read_traffic_summary(cfg.name, kernels[dom]["name"]),
                "launch_seconds": kernels[dom]["seconds"], "algorithmic_bytes": kernels[dom]["bytes"]}
    stage_bytes = bytes_gather + bytes_agg
    # the same stage priced as two separate passes (copy every row of S_{H-1}, then read every row of X back once): what a
    # gather followed by an aggregation over X has to move at least; the stage above moves less because a row goes
    # from the table through the aggregation's registers into X
    two_pass_bytes = nH * (4 + 2 * 4 * cfg.dim) + nH * 4 * cfg.dim + EHm1 * 4 + (nHm1 + 1) * 4 + nHm1 * 4 * cfg.dim
    stage = {"gather_plus_aggregate_GBps": stage_bytes / (t_gather + t_agg) / 1e9,
             "frac_of_peak": stage_bytes / (t_gather + t_agg) / 1e9 / HBM_PEAK_GBS,
             "features": "one pass (aggregation reads the table, writes the new vertices' rows of X)" if one_pass else
                         "two passes (gather copies every row, aggregation reads X)",
             "two_pass_bytes": two_pass_bytes, "two_pass_equivalent_GBps": two_pass_bytes / (t_gather + t_agg) / 1e9,
             "share_of_single_stream_step": (t_gather + t_agg) / (wall_single / K)}

    # ---- CPU baseline: the checker as it stands, on the host cores, on a bounded sample of the same steps
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import zg_oracle
        cores = max(1, min(16, len(os.sched_getaffinity(0))))
        t_host = time.perf_counter()
        og = zg_oracle.Graph(g.offsets.cpu().numpy(), g.indices.cpu().numpy())
        feat_h = feat.cpu().numpy()
        seeds_h = [b.cpu().numpy() for b in batches[Wm:]]
        log(f"[bench] host copies of graph and feature table for the checker ({time.perf_counter() - t_host:.1f}s)")

        def one(s):
            zg_oracle.step(og, seeds_h[s % K], cfg.fanouts, keys[Wm + s % K], feat_h)
            return s
        # rounds of `cores` independent steps until the time budget is used (the step list wraps around if it is short)
        done = 0
        t_cpu0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            while time.perf_counter() - t_cpu0 < args.cpu_seconds:
                list(ex.map(one, range(done, done + cores)))
                done += cores
        t_cpu = time.perf_counter() - t_cpu0
        t1 = time.perf_counter()
        n1 = 0
        while n1 < min(K, 8) and time.perf_counter() - t1 < 5.0:
            one(n1)
            n1 += 1
        single = n1 / (time.perf_counter() - t1)
        cpu = {"value": done / t_cpu, "unit": "mini-batches/s", "cores": cores, "kind": "oracle",
               "single_thread_value": single,
               "sample": f"{done} steps (the {K} timed steps of {cfg.name}, repeated in order), {cores} threads over independent "
                         f"steps, {t_cpu:.1f}s"}

    out = {
        "metric": "sampled mini-batches/sec (sample+relabel+gather+mean-agg)",
        "value": value, "unit": "mini-batches/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 ids / f32 features", "data": "synthetic",
        "config": {"workload": cfg.name, "graph": f"{cfg.kind} |V|={g.num_nodes} |E|={g.num_edges}",
                   "offsets": str(g.offsets.dtype).replace("torch.", ""), "feat_dim": cfg.dim, "batch": cfg.batch,
                   "fanouts": list(cfg.fanouts), "envelope": env_mode, "launch": ("kernels launched one by one (--eager)" if args.eager else "1 hipGraph replay per step"),
                   "pipeline": f"{pipeline} plan(s) on {pipeline} stream(s), steps issued round-robin",
                   "host_syncs_in_timed_region": 1},
        "single_stream": {"value": K / wall_single, "ms_per_step": wall_single / K * 1e3},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "stage": stage,
        "sizes": {"n_mean": n_steps.mean(0).tolist(), "n_min": n_steps.min(0).tolist(), "n_max": n_steps.max(0).tolist(),
                  "E_mean": E_steps.mean(0).tolist(), "node_cap": [int(info.node_cap[h]) for h in range(H + 1)],
                  "maxsg_nodes": [int(info.maxsg_nodes[h]) for h in range(H + 1)],
                  "model_mean": [float(info.model_mean[h]) for h in range(H + 1)],
                  "model_sigma": [float(info.model_sigma[h]) for h in range(H + 1)],
                  # the distribution of the last hop's size over the timed steps (the paper's appendix B histogram):
                  # ten equal bins between min and max, the spread (max - min) / mean, and the cap's headroom over the max
                  "n_H_histogram": np.histogram(n_steps[:, H], bins=10)[0].tolist(),
                  "n_H_spread": float((n_steps[:, H].max() - n_steps[:, H].min()) / n_steps[:, H].mean()),
                  "n_H_std_over_mean": float(n_steps[:, H].std() / n_steps[:, H].mean()),
                  "cap_over_max": float(info.node_cap[H] / n_steps[:, H].max())},
        "memory": {"envelope_bytes": int(info.envelope_bytes), "scratch_bytes": int(info.scratch_bytes),
                   "maxsg_envelope_bytes": int(info.maxsg_envelope_bytes), "exact_bytes_mean": float(exact.mean()),
                   "exact_bytes_max": float(exact.max()), "envelope_over_exact_mean": float(info.envelope_bytes / exact.mean()),
                   "maxsg_over_envelope": float(info.maxsg_envelope_bytes / info.envelope_bytes),
                   "overflow_steps": int((recs[:, 1] != 0).sum())},
        "paper_context": "ZeroGNN reports up to 5.28x end-to-end speedup over DGL and ~100% GPU execution fraction on "
                         "NVIDIA A100 80GB (CUDA 11.7); ratios only, no absolute throughput",
    }
    if fused is not None:
        out["fused_input"] = fused
    if auto_fb is not None:
        out["auto_fallback"] = auto_fb
    if gm is not None:
        ginfo, t_gm = gm
        out["graph_model_envelope"] = {
            "node_cap": [int(ginfo.node_cap[h]) for h in range(H + 1)], "envelope_bytes": int(ginfo.envelope_bytes),
            "envelope_over_exact_mean": float(ginfo.envelope_bytes / exact.mean()),
            "cap_over_max": [float(ginfo.node_cap[h] / n_steps[:, h].max()) for h in range(1, H + 1)],
            "would_overflow_steps": int((n_steps[:, 1:] > np.array([ginfo.node_cap[h] for h in range(1, H + 1)])).any(1).sum()),
            "model_seconds": t_gm}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
