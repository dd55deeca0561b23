"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI binding and compare
every output with the CPU checker on the same seeded inputs."""
import numpy as np
import torch

from paper_2605_29346_amd import zg

AGG_RTOL = 1e-5  # fp32 mean aggregation: |gpu - ref| <= 1e-5 * max(|ref|, mean over the row of |x|)


def to_host_graph(oracle, g):
    return oracle.Graph(g.offsets.cpu().numpy(), g.indices.cpu().numpy())


def compare_blocks(res, ref, label=""):
    """Bit-exact comparison of counts, vertex list and every hop's block CSR."""
    H = len(ref.E)
    assert res.flags == 0, f"{label}: status flags {res.flags:#x}"
    assert res.n == ref.n, f"{label}: n {res.n} != {ref.n}"
    assert res.E == ref.E, f"{label}: E {res.E} != {ref.E}"
    assert res.n_exact[1:] == ref.n[1:], f"{label}: n_exact"
    assert np.array_equal(res.S, ref.S), f"{label}: S differs"
    for h in range(H):
        assert np.array_equal(res.row_ptr[h], ref.row_ptr[h]), f"{label}: row_ptr[{h}]"
        assert np.array_equal(res.nbr_gid[h], ref.nbr_gid[h]), f"{label}: nbr_gid[{h}]"
        assert np.array_equal(res.col[h], ref.col[h]), f"{label}: col[{h}]"


def agg_error(oracle, got, ref_agg, row_ptr, col, X):
    """max over elements of |got - ref| / max(|ref|, mean_row |x|) (0/0 counts as 0)."""
    denom = np.maximum(np.abs(ref_agg), oracle.aggregate_mean(row_ptr, col, np.abs(X)))
    err = np.abs(got.astype(np.float64) - ref_agg.astype(np.float64))
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(denom > 0, err / denom, np.where(err == 0, 0.0, np.inf))
    return float(rel.max()) if rel.size else 0.0


def compare_features(oracle, res, ref, feat_host, label=""):
    X_ref = oracle.gather(feat_host, ref.S)
    assert np.array_equal(res.X.view(np.uint32), X_ref.view(np.uint32)), f"{label}: gathered rows differ"
    agg_ref = oracle.aggregate_mean(ref.row_ptr[-1], ref.col[-1], X_ref)
    assert res.agg.shape == agg_ref.shape
    e = agg_error(oracle, res.agg, agg_ref, ref.row_ptr[-1], ref.col[-1], X_ref)
    assert e <= AGG_RTOL, f"{label}: aggregation error {e}"
    return e


def run_and_compare(oracle, g, feat, seeds, fanouts, key, *, env=None, plan=None, og=None, replace=False, label=""):
    """One step on the GPU (new plan unless given) against the checker; returns (plan, result, reference)."""
    dev_g = None
    if plan is None:
        dev_g = zg.Graph(g.offsets.cuda(), g.indices.cuda())
        flags = zg.PLAN_REPLACE if replace else 0
        env = env or zg.make_envelope(zg.ENV_MAX, flags=flags)
        plan = zg.Plan(dev_g, fanouts, len(seeds), env, feat_dim=0 if feat is None else feat.shape[1])
        if feat is not None:
            plan.bind_features(feat.cuda())
    og = og or to_host_graph(oracle, g)
    seeds_d = torch.as_tensor(np.asarray(seeds, dtype=np.int32)).cuda()
    plan.step(seeds_d, key)
    res = plan.read_step()
    ref = og.sample_blocks(np.asarray(seeds, dtype=np.int32), fanouts, key, with_replacement=replace)
    compare_blocks(res, ref, label)
    if feat is not None:
        compare_features(oracle, res, ref, feat.cpu().numpy(), label)
    return plan, res, ref
