#!/usr/bin/env python3
"""Throughput of the whole mini-batch construction step on one MI355X.

One "step" = one pass of the hot path (sample -> dedup/relabel -> block CSR -> gather -> mean
aggregation) over one synthetic mini-batch, issued through the C-ABI library as one ingest kernel
plus one hipGraph replay, with no host synchronisation between steps.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload medium_dense] [--env model|max]

Besides the headline value the line carries
  roofline     - the dominant kernel of the step (gather or aggregate): algorithmic bytes per launch
                 / its average launch duration, measured here with events on the launch stream,
                 against MI355X's 8 TB/s HBM peak;
  cpu_baseline - the CPU checker (oracle/, untuned) timed on this machine's host cores on a bounded
                 sample of the same steps.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic_summary(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, if there is one
    (profiles/hbm_traffic_<workload>.txt, lines `<kernel> <fetch_bytes> <write_bytes>`)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 3 and parts[0] == kernel:
            try:
                return float(parts[1]) + float(parts[2])
            except ValueError:
                return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="medium_dense")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only; invalid as a result)")
    ap.add_argument("--env", default="model", choices=["model", "max", "graph"],
                    help="envelope of the plans: the paper's Lemma 1 from the degree histogram (default), the worst case, or "
                         "explicit caps from the graph-aware size model")
    ap.add_argument("--eager", action="store_true", help="plans launch their kernels one by one instead of replaying a hipGraph "
                    "(a comparison; the default and the reported configuration is the captured graph)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--no-fused", action="store_true", help="skip the extra pass with ZG_PLAN_FUSED_INPUT plans")
    ap.add_argument("--pipeline", type=int, default=4,
                    help="independent plans replayed round-robin on their own streams (consecutive mini-batches do not "
                         "depend on each other); 1 = strictly one step after the other")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a single-GPU path (no sharding, no collectives); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2605_29346_amd import workloads as W
    from paper_2605_29346_amd import zg

    from paper_2605_29346_amd import build as zg_build
    if not os.path.exists(zg_build.LIB):  # load what is built; build only if nothing is
        zg_build.build(force=True)
    zg.lib()  # fails loudly if the HIP library still cannot be loaded: there is no other path
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"

    cfg = W.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = cfg.scaled(args.scale)
    K, Wm = args.steps, args.warmup

    t0 = time.time()
    g = cfg.build_graph(device=dev)
    torch.cuda.synchronize()
    log(f"[bench] graph {cfg.name}: |V|={g.num_nodes} |E|={g.num_edges} ({time.time() - t0:.1f}s)")
    t0 = time.time()
    feat = W.feature_table(g.num_nodes, cfg.dim, cfg.feat_seed, device=dev)
    pool = cfg.seed_pool(g)
    batches = [pool.batch_for(s).contiguous() for s in range(K + Wm)]
    keys = [cfg.key_for(s) for s in range(K + Wm)]
    torch.cuda.synchronize()
    log(f"[bench] features {tuple(feat.shape)} + {len(batches)} seed batches ({time.time() - t0:.1f}s)")

    dg = zg.Graph(g.offsets, g.indices)
    H = len(cfg.fanouts)

    def make_plan(mode, flags=0):
        flags |= zg.PLAN_EAGER if args.eager else 0
        if mode == "graph":
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

    env_mode = args.env
    plan = make_plan(env_mode)
    cur = torch.cuda.current_stream()
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

    # extra (not the headline): the same steps with plans that materialise only the frontier's rows of X and
    # aggregate straight from the feature table (what the first GraphSAGE layer needs)
    fused = None
    if not args.no_fused:
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
    auto_fb = None
    if not args.no_fused and env_mode != "max":
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
    ginfo = dg.plan_query(cfg.fanouts, cfg.batch, genv, feat_dim=cfg.dim)

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
    X = plan.view_X()
    aggv = plan.view_agg()
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

    t_gather = time_kernel(lambda: plan.gather(feat, X[:, :cfg.dim]))
    t_agg = time_kernel(lambda: plan.aggregate_mean(H - 1, X[:, :cfg.dim], aggv[:, :cfg.dim]))
    bytes_gather = nH * (4 + 2 * 4 * cfg.dim)
    bytes_agg = nH * 4 * cfg.dim + EHm1 * 4 + (nHm1 + 1) * 4 + nHm1 * 4 * cfg.dim
    bytes_agg_noreuse = EHm1 * 4 * cfg.dim + EHm1 * 4 + (nHm1 + 1) * 4 + nHm1 * 4 * cfg.dim
    kernels = {
        "gather": {"seconds": t_gather, "bytes": bytes_gather, "GBps": bytes_gather / t_gather / 1e9,
                   "name": "k_gather"},
        # `bytes` is the compulsory figure (every input row once); without cache reuse every edge fetches its row
        "aggregate": {"seconds": t_agg, "bytes": bytes_agg, "GBps": bytes_agg / t_agg / 1e9, "name": "k_aggregate",
                      "bytes_without_reuse": bytes_agg_noreuse, "GBps_without_reuse": bytes_agg_noreuse / t_agg / 1e9},
    }
    dom = max(kernels, key=lambda k: kernels[k]["seconds"])
    roofline = {"bound": "hbm", "kernel": kernels[dom]["name"], "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kernels[dom]["GBps"] / HBM_PEAK_GBS,
                "traffic": read_traffic_summary(cfg.name, kernels[dom]["name"]),
                "launch_seconds": kernels[dom]["seconds"], "algorithmic_bytes": kernels[dom]["bytes"]}
    stage_bytes = bytes_gather + bytes_agg
    stage = {"gather_plus_aggregate_GBps": stage_bytes / (t_gather + t_agg) / 1e9,
             "frac_of_peak": stage_bytes / (t_gather + t_agg) / 1e9 / HBM_PEAK_GBS,
             "share_of_single_stream_step": (t_gather + t_agg) / (wall_single / K)}

    # ---- CPU baseline: the checker as it stands, on the host cores, on a bounded sample of the same steps
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import zg_oracle
        cores = max(1, min(16, len(os.sched_getaffinity(0))))
        og = zg_oracle.Graph(g.offsets.cpu().numpy(), g.indices.cpu().numpy())
        feat_h = feat.cpu().numpy()
        seeds_h = [b.cpu().numpy() for b in batches[Wm:]]

        def one(s):
            zg_oracle.step(og, seeds_h[s], cfg.fanouts, keys[Wm + s], feat_h)
            return s
        done = 0
        t_cpu0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            while done < K and time.perf_counter() - t_cpu0 < args.cpu_seconds:
                chunk = list(range(done, min(K, done + cores)))
                list(ex.map(one, chunk))
                done += len(chunk)
        t_cpu = time.perf_counter() - t_cpu0
        t1 = time.perf_counter()
        n1 = 0
        while n1 < min(K, 8) and time.perf_counter() - t1 < 5.0:
            one(n1)
            n1 += 1
        single = n1 / (time.perf_counter() - t1)
        cpu = {"value": done / t_cpu, "unit": "mini-batches/s", "cores": min(cores, done), "kind": "oracle",
               "single_thread_value": single,
               "sample": f"first {done} of the {K} timed steps of {cfg.name}, {cores} threads over independent steps, "
                         f"{t_cpu:.1f}s"}

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
        "fused_input": fused,
        "auto_fallback": auto_fb,
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
        "graph_model_envelope": {"node_cap": [int(ginfo.node_cap[h]) for h in range(H + 1)],
                                 "envelope_bytes": int(ginfo.envelope_bytes),
                                 "envelope_over_exact_mean": float(ginfo.envelope_bytes / exact.mean()),
                                 "cap_over_max": [float(ginfo.node_cap[h] / n_steps[:, h].max()) for h in range(1, H + 1)],
                                 "would_overflow_steps": int((n_steps[:, 1:] > np.array([ginfo.node_cap[h] for h in range(1, H + 1)])).any(1).sum()),
                                 "model_seconds": t_gm},
        "paper_context": "ZeroGNN reports up to 5.28x end-to-end speedup over DGL and ~100% GPU execution fraction on "
                         "NVIDIA A100 80GB (CUDA 11.7); ratios only, no absolute throughput",
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
