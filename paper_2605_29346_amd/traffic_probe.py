"""A short run of the hot path for counter collection: a few steps of one workload plus one plain
streaming kernel of known size (dst = src * 1 over CALIB_BYTES of fp32) that calibrates the HBM
counters.  Meant to be run under `rocprofv3 --pmc FETCH_SIZE` and, separately, `--pmc WRITE_SIZE`:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o fetch -- python3 -m paper_2605_29346_amd.traffic_probe
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir> -o write -- python3 -m paper_2605_29346_amd.traffic_probe
    python3 -m paper_2605_29346_amd.profile_summary pmc <dir>/fetch_counter_collection.csv <dir>/write_counter_collection.csv
"""
import argparse
import sys

CALIB_ELEMS = 96 * 1024 * 1024 + 4096  # fp32 elements of the calibration kernel (an unusual grid size, easy to find)
CALIB_BYTES = CALIB_ELEMS * 4          # it reads CALIB_BYTES and writes CALIB_BYTES


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="medium_dense")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    args = ap.parse_args()
    import torch
    from . import workloads as W
    from . import zg
    cfg = W.CONFIGS[args.workload]
    g = cfg.build_graph(device="cuda")
    feat = W.feature_table(g.num_nodes, cfg.dim, cfg.feat_seed, device="cuda")
    pool = cfg.seed_pool(g)
    dg = zg.Graph(g.offsets, g.indices)
    plan = zg.Plan(dg, cfg.fanouts, cfg.batch, zg.make_envelope(zg.ENV_MODEL), feat_dim=cfg.dim)
    plan.bind_features(feat)
    batches = [pool.batch_for(s).contiguous() for s in range(args.steps + args.warmup)]
    src = torch.ones(CALIB_ELEMS, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for s, b in enumerate(batches):
        plan.step(b, cfg.key_for(s))
    torch.cuda.synchronize()
    for _ in range(3):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    n, E, _, flags = [t.cpu().tolist() for t in plan.view_counts()]
    print(f"workload {cfg.name}: last step n={n} E={E} flags={flags} calib_bytes={CALIB_BYTES}", file=sys.stderr)


if __name__ == "__main__":
    main()
