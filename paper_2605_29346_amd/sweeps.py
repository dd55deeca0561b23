"""The parameter sweeps of the paper's evaluation, re-run on the synthetic stand-in for its Reddit setting
(the medium-dense workload): batch size 64..4096, sampling depth 2..5 hops, memory of the envelope against
the worst-case reservation per depth, and launch over-provisioning (+20 % .. +180 % capacity at fixed work).
Prints markdown tables.

    python -m paper_2605_29346_amd.sweeps [--workload medium_dense] [--steps 60] [--which batch,depth,overalloc]
"""
import argparse
import dataclasses
import sys
import time


def run_steps(plans, streams, batches, keys, warm, steps):
    import torch
    P = len(plans)
    for s in range(warm):
        plans[s % P].step(batches[s % len(batches)], keys[s], streams[s % P])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(warm, warm + steps):
        plans[s % P].step(batches[s % len(batches)], keys[s], streams[s % P])
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="medium_dense")
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--which", default="batch,depth,overalloc")
    args = ap.parse_args()
    import numpy as np
    import torch
    from . import workloads as W
    from . import zg

    base = W.CONFIGS[args.workload]
    g = base.build_graph(device="cuda")
    feat = W.feature_table(g.num_nodes, base.dim, base.feat_seed, device="cuda")
    dg = zg.Graph(g.offsets, g.indices)
    streams = [zg.new_stream() for _ in range(4)]
    cur = [torch.cuda.current_stream().cuda_stream]
    K, Wm = args.steps, args.warmup
    which = set(args.which.split(","))
    print(f"graph {base.name}: |V|={g.num_nodes} |E|={g.num_edges}, feature dim {base.dim}\n")

    def measure(cfg, env, pipelined=True):
        pool = cfg.seed_pool(g)
        batches = [pool.batch_for(s).contiguous() for s in range(K + Wm)]
        keys = [cfg.key_for(s) for s in range(K + Wm)]
        plans = []
        for _ in range(4 if pipelined else 1):
            p = zg.Plan(dg, cfg.fanouts, cfg.batch, env, feat_dim=cfg.dim)
            p.bind_features(feat)
            plans.append(p)
        t1 = run_steps(plans[:1], cur, batches, keys, Wm, K)
        tp = run_steps(plans, streams, batches, keys, Wm, K) if pipelined else t1
        flags = 0
        for p in plans:
            flags |= int(p.view_counts()[3].cpu()[0]) & 0xFFFFFFFF
        n = [int(x) for x in plans[0].view_counts()[0].cpu().tolist()]
        info = plans[0].info
        for p in plans:
            p.close()
        return t1, tp, flags, n, info

    if "batch" in which:
        print("### batch-size sweep (fanouts fixed)\n")
        print("| batch | us/step, one stream | mini-batches/s, one stream | mini-batches/s, 4 plans | seeds/s, 4 plans | n_H of the last step |")
        print("|---|---|---|---|---|---|")
        for B in (64, 128, 256, 512, 1024, 2048, 4096):
            cfg = dataclasses.replace(base, batch=B)
            t1, tp, flags, n, _ = measure(cfg, zg.make_envelope(zg.ENV_MAX))
            assert flags == 0
            print(f"| {B} | {t1 * 1e6:.1f} | {1 / t1:.0f} | {1 / tp:.0f} | {B / tp:.3g} | {n[-1]} |", flush=True)
        print()

    if "depth" in which:
        print("### depth sweep (batch fixed, fanout 10 beyond the configured hops) and envelope memory per depth\n")
        print("| hops | fanouts | us/step, one stream | mini-batches/s, 4 plans | n_H | envelope MB (model, 20 % margin) | worst-case MB | worst case / envelope | overflowed |")
        print("|---|---|---|---|---|---|---|---|---|")
        for H in (2, 3, 4, 5):
            fan = tuple(list(base.fanouts) + [10] * 5)[:H]
            cfg = dataclasses.replace(base, fanouts=fan)
            t1, tp, flags, n, info = measure(cfg, zg.make_envelope(zg.ENV_MODEL))
            print(f"| {H} | {list(fan)} | {t1 * 1e6:.1f} | {1 / tp:.0f} | {n[-1]} | {info.envelope_bytes / 1e6:.0f} | "
                  f"{info.maxsg_envelope_bytes / 1e6:.0f} | {info.maxsg_envelope_bytes / info.envelope_bytes:.2f} | "
                  f"{'yes' if flags else 'no'} |", flush=True)
        print()

    if "overalloc" in which:
        print("### launch over-provisioning at fixed work (caps = realised sizes times the factor)\n")
        cfg = base
        # realised sizes from a pilot run on the worst-case envelope
        pool = cfg.seed_pool(g)
        pilot = zg.Plan(dg, cfg.fanouts, cfg.batch, zg.make_envelope(zg.ENV_MAX), feat_dim=0)
        nmax = np.zeros(len(cfg.fanouts) + 1, dtype=np.int64)
        for s in range(K + Wm):
            pilot.step(pool.batch_for(s).contiguous(), cfg.key_for(s))
            torch.cuda.synchronize()
            nmax = np.maximum(nmax, pilot.view_counts()[0].cpu().numpy())
        pilot.close()
        print("| capacity over the largest realised size | node caps | us/step, one stream | vs +20 % |")
        print("|---|---|---|---|")
        ref = None
        for extra in (0.2, 0.6, 1.0, 1.4, 1.8):
            caps = [0] + [int(x * (1 + extra)) + 1 for x in nmax[1:]]
            t1, _, flags, n, info = measure(cfg, zg.make_envelope(zg.ENV_EXPLICIT, node_caps=caps), pipelined=False)
            assert flags == 0
            ref = ref or t1
            print(f"| +{extra * 100:.0f} % | {[int(info.node_cap[h]) for h in range(len(cfg.fanouts) + 1)]} | {t1 * 1e6:.1f} | "
                  f"{t1 / ref:.3f} |", flush=True)
        print()


if __name__ == "__main__":
    sys.exit(main())
