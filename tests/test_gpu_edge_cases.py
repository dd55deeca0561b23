"""GPU parity on the degenerate and extreme shapes of the method: no edges at all, a single seed, every
vertex a seed, the maximum number of hops, fanout 64 on a six-figure degree, vertex counts that are not a
multiple of 32, and every tile-size variant of the chained-scan kernels (forced through the envelope's max_tickets knob)."""
import os

import numpy as np
import pytest
import torch

from paper_2605_29346_amd import workloads as W
from paper_2605_29346_amd import zg
from gpu_util import agg_error, compare_blocks, run_and_compare, to_host_graph

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    zg.lib()


def _csr(rows, n):
    off = np.zeros(n + 1, dtype=np.int64)
    for v, r in rows.items():
        off[v + 1] = len(r)
    off = np.cumsum(off)
    idx = np.concatenate([np.asarray(sorted(rows[v]), dtype=np.int32) for v in sorted(rows)] or [np.zeros(0, np.int32)])
    return W.Graph(n, torch.as_tensor(off), torch.as_tensor(idx.astype(np.int32)))


def test_graph_without_edges(oracle):
    n = 1000
    g = W.Graph(n, torch.zeros(n + 1, dtype=torch.int32), torch.zeros(0, dtype=torch.int32))
    feat = W.feature_table(n, 8, 1)
    seeds = np.arange(5, 45, dtype=np.int32)
    _, res, ref = run_and_compare(oracle, g, feat, seeds, (3, 3), 7)
    assert res.n == [40, 40, 40] and res.E == [0, 0] and np.all(res.agg == 0)


def test_single_seed_and_single_vertex(oracle):
    g = W.rmat_graph(5000, 90_000, 2)
    feat = W.feature_table(5000, 12, 1)
    deg = np.diff(g.offsets.numpy())
    run_and_compare(oracle, g, feat, np.array([int(np.argmax(deg))], dtype=np.int32), (5, 5, 5), 3)
    run_and_compare(oracle, g, feat, np.array([int(np.argmin(deg))], dtype=np.int32), (5, 5, 5), 3)
    one = W.Graph(1, torch.tensor([0, 1], dtype=torch.int32), torch.tensor([0], dtype=torch.int32))  # a self-loop
    _, res, _ = run_and_compare(oracle, one, torch.ones(1, 4), np.array([0], dtype=np.int32), (2, 2), 1)
    assert res.n == [1, 1, 1] and res.E == [1, 1] and np.all(res.col[0] == 0)


@pytest.mark.parametrize("nodes", [31, 32, 33, 1023, 4097])
def test_every_vertex_is_a_seed(oracle, nodes):
    g = W.rmat_graph(nodes, nodes * 12, nodes)
    feat = W.feature_table(nodes, 4, 1)
    seeds = np.random.RandomState(nodes).permutation(nodes).astype(np.int32)
    _, res, _ = run_and_compare(oracle, g, feat, seeds, (4, 2), 11)
    assert res.n == [nodes, nodes, nodes]  # nothing new can be discovered


def test_maximum_hops(oracle):
    g = W.rmat_graph(20_000, 200_000, 5)
    feat = W.feature_table(20_000, 8, 1)
    seeds = W.SeedPool(g, 16, 1).batch_for(0).numpy()
    _, res, _ = run_and_compare(oracle, g, feat, seeds, (2,) * 8, 13)
    assert len(res.E) == 8
    dg = zg.Graph(g.offsets.cuda(), g.indices.cuda())
    with pytest.raises(zg.ZgError):
        zg.Plan(dg, (2,) * 9, 16)


def test_fanout_64_on_a_huge_row(oracle):
    # one vertex adjacent to 150k others, fanout 64 (the widest lane group) and fanout 63, with and without replacement
    n = 200_000
    rnd = np.random.RandomState(3)
    hub_nb = np.sort(rnd.choice(n, 150_000, replace=False)).astype(np.int32)
    rows = {0: hub_nb.tolist()}
    for v in range(1, 400):
        rows[v] = sorted(set(rnd.randint(0, n, size=rnd.randint(0, 130)).tolist()))
    g = _csr(rows, n)
    feat = W.feature_table(n, 4, 2)
    seeds = np.arange(0, 300, dtype=np.int32)
    for fan in ((64, 2), (63, 64)):
        for key in (1, 2):
            run_and_compare(oracle, g, feat, seeds, fan, key)
        run_and_compare(oracle, g, feat, seeds, fan, 5, replace=True)


@pytest.mark.parametrize("max_tickets", [1, 2, 4, 16, 64])
def test_all_tile_variants_of_the_chained_scans(oracle, max_tickets):
    # tiny ticket budgets force several tiles of old rows per ticket and ranking tiles of up to 8 words per lane, each
    # holding many batches of 256 new rows
    g = W.rmat_graph(600_000, 3_000_000, 17)
    feat = W.feature_table(600_000, 4, 2)
    og = to_host_graph(oracle, g)
    pool = W.SeedPool(g, 3000, 5)
    plan = None
    for s in range(2):
        plan, res, ref = run_and_compare(oracle, g, feat, pool.batch_for(s).numpy(), (6, 5, 3), 40 + s, plan=plan, og=og,
                                         env=zg.make_envelope(zg.ENV_MAX, max_tickets=max_tickets))
    info = plan.info
    words = -(-600_000 // 32)
    assert info.grid_compact <= max(max_tickets, -(-words // 8192))
    # up to 256 old rows per ticket, ranking tiles of at most 8192 words
    assert info.grid_sample[2] <= max(max_tickets, -(-info.node_cap[1] // 256)) + max(max_tickets, -(-words // 8192))


def test_sparse_launch_over_a_long_bitmap_takes_16_words_per_lane(oracle):
    # a handful of seeds on a 600 k-vertex graph: the launches that rank hop 0's and hop 1's few discoveries need one or two
    # tickets for their rows, so their ranking tiles grow to 16384 words (16 per lane: the second instantiation of the
    # hop kernel); the last tile reaches past the bitmap's last word into its zero padding
    g = W.rmat_graph(600_000, 3_000_000, 17)
    feat = W.feature_table(600_000, 8, 2)
    og = to_host_graph(oracle, g)
    pool = W.SeedPool(g, 6, 11)
    plan = None
    for s in range(3):
        plan, res, ref = run_and_compare(oracle, g, feat, pool.batch_for(s).numpy(), (4, 3, 3), 70 + s, plan=plan, og=og,
                                         env=zg.make_envelope(zg.ENV_MAX))
    words = -(-600_000 // 32)
    # launch 1: its old rows' tickets plus ranking tiles of 16384 words
    assert plan.info.grid_sample[1] <= 1 + -(-words // 16384) + 1
    assert ref.n[-1] > 6
    # the same launches with a cap that cuts into the rows a 16-word tile ranks: flagged, and the rows kept are a prefix
    seeds = pool.batch_for(2).numpy()
    caps = [0, ref.n[1], ref.n[2] - 3, ref.n[3]]
    tight = zg.Plan(zg.Graph(g.offsets.cuda(), g.indices.cuda()), (4, 3, 3), 6, zg.make_envelope(zg.ENV_EXPLICIT, node_caps=caps), feat_dim=0)
    tight.step(torch.as_tensor(seeds).cuda(), 72)
    torch.cuda.synchronize()
    n, E, n_exact, flags = [t.cpu().numpy() for t in tight.view_counts()]
    assert int(flags[0]) & zg.FLAG_HOP_OVERFLOW(1)
    assert n[2] == ref.n[2] - 3 and n_exact[2] == ref.n[2]
    assert np.array_equal(tight.view_S()[: n[2]].cpu().numpy(), ref.S[: n[2]])


def test_randomised_configurations(oracle):
    # 40 random (graph, batch, hops, fanouts, feature width, envelope mode, replacement) draws, two steps each
    # (ZG_FUZZ_TRIALS runs more of them, ZG_FUZZ_SEED another sequence)
    rnd = np.random.RandomState(int(os.environ.get("ZG_FUZZ_SEED", "20260529")))
    for trial in range(int(os.environ.get("ZG_FUZZ_TRIALS", "40"))):
        if trial and trial % 50 == 0:
            print(f"[fuzz] {trial} trials done", flush=True)
        nodes = int(rnd.choice([50, 333, 2048, 7001, 40_000, 150_000]))
        avg_deg = float(rnd.choice([0.5, 3, 20, 120]))
        draws = max(64, int(nodes * avg_deg))
        i64 = bool(rnd.randint(2))
        g = W.rmat_graph(nodes, draws, 1000 + trial, offsets_dtype=torch.int64 if i64 else torch.int32)
        H = int(rnd.randint(1, 5))
        fan = tuple(int(rnd.choice([1, 2, 3, 5, 8, 13, 16, 25, 40, 64])) for _ in range(H))
        batch = int(min(nodes, rnd.choice([1, 7, 64, 300, 1024])))
        dim = int(rnd.choice([1, 4, 10, 32, 100, 257]))
        replace = bool(rnd.randint(4) == 0)
        mode = [zg.ENV_MAX, zg.ENV_MODEL][int(rnd.randint(2))]
        feat = W.feature_table(nodes, dim, trial)
        og = to_host_graph(oracle, g)
        dg = zg.Graph(g.offsets.cuda(), g.indices.cuda(), validate=True)
        flags = (zg.PLAN_REPLACE if replace else 0) | (zg.PLAN_FUSED_INPUT if rnd.randint(3) == 0 else 0)
        flags |= [0, zg.PLAN_X_ONE_PASS, zg.PLAN_X_TWO_PASS][int(rnd.randint(3))]  # who writes the new vertices' rows of X
        auto = mode == zg.ENV_MODEL and rnd.randint(2) == 0  # the twin's gated kernels redo an overflowed step
        flags |= zg.PLAN_AUTO_FALLBACK if auto else 0
        try:
            plan = zg.Plan(dg, fan, batch, zg.make_envelope(mode, flags=flags), feat_dim=dim)
        except zg.ZgError as e:  # a hop's edge capacity reaching 2^31 is refused, nothing else may be
            assert "2^31" in str(e), str(e)
            continue
        plan.bind_features(feat.cuda())
        pool = W.SeedPool(g, batch, trial)
        label = f"trial {trial}: V={nodes} draws={draws} i64={i64} fan={fan} B={batch} dim={dim} replace={replace} mode={mode} flags={flags}"
        for s in range(2):
            seeds = pool.batch_for(s).numpy()
            plan.step(torch.as_tensor(seeds).cuda(), 77 + s)
            res = plan.read_step()
            ref = og.sample_blocks(seeds, fan, 77 + s, with_replacement=replace)
            if auto:
                assert int(plan.view_active().item()) == (1 if res.flags & 0xFF else 0), label
            if res.flags:  # the model envelope may be too tight on these odd little graphs: flagged, and redone if armed
                assert mode == zg.ENV_MODEL and (res.flags & 0xFF), label
                plan.overflow_clear()
                if not auto:
                    continue
                res = plan.safe_view().read_step()
                label += " (twin)"
            compare_blocks(res, ref, label)
            X_ref = oracle.gather(feat.numpy(), ref.S)
            xr = ref.n[-2] if flags & zg.PLAN_FUSED_INPUT else ref.n[-1]
            assert np.array_equal(res.X.view(np.uint32), X_ref[:xr].view(np.uint32)), label
            agg_ref = oracle.aggregate_mean(ref.row_ptr[-1], ref.col[-1], X_ref)
            assert agg_error(oracle, res.agg, agg_ref, ref.row_ptr[-1], ref.col[-1], X_ref) <= 1e-5, label
        plan.close()


def test_worked_example_from_the_published_known_answer(oracle):
    # vertex 0, slot 0, hop 0, key 0 is the all-zero Philox input (published output 6627e8d5 e169c58d ...): the draw is
    # 0xe169c58d6627e8d5 = 0.88052 * 2^64, so one slot over d neighbors lands on position floor(0.88052 d)
    x = 0xE169C58D6627E8D5
    for d in (5, 3, 100, 1000):
        expect = (x * d) >> 64
        off = np.zeros(d + 2, dtype=np.int64)
        off[1:] = d
        g = W.Graph(d + 1, torch.as_tensor(off), torch.arange(1, d + 1, dtype=torch.int32))
        _, res, _ = run_and_compare(oracle, g, None, np.array([0], dtype=np.int32), (1,), 0)
        assert res.nbr_gid[0].tolist() == [expect + 1] and res.S.tolist() == [0, expect + 1]
