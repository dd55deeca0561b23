"""CPU-only checks of the C-ABI library: it loads, exports what include/zg.h declares, and its
host-side planner (envelope model of Lemma 1 / appendix A, caps, layout) is right."""
import ctypes
import math
import os
import re
import subprocess

import numpy as np
import pytest

from paper_2605_29346_amd import zg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "zg.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(zg_[a-z_0-9]+)\s*\(", hdr))
    assert {"zg_graph_create", "zg_plan", "zg_step", "zg_gather", "zg_aggregate_mean", "zg_overflow_flag"} <= declared
    L = zg.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in zg.h but not exported"
    assert declared == set(zg.EXPORTS)


def test_struct_sizes_match_header_layout(tmp_path):
    # compile the header with gcc (it is plain C) and compare sizeof with the ctypes mirrors
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "zg.h"\nint main(void){printf("%zu %zu %zu\\n", '
                   'sizeof(zg_envelope), sizeof(zg_plan_info), sizeof(zg_outputs));return 0;}\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [ctypes.sizeof(zg.Envelope), ctypes.sizeof(zg.PlanInfo), ctypes.sizeof(zg.Outputs)]


def test_normal_quantile_against_scipy_and_appendix_values():
    from scipy.stats import norm
    for p in (0.5, 0.9, 0.975, 0.999, 1e-6, 1 - 1e-9):
        assert abs(zg.normal_quantile(p) - norm.ppf(p)) < 1e-9
    # z_p^(m) = Phi^-1(p^(1/m)) (appendix A)
    assert abs(zg.normal_quantile(0.999 ** (1 / 1000)) - 4.753) < 2e-3
    assert abs(zg.normal_quantile(0.9999 ** (1 / 500)) - 5.069) < 2e-3


def test_envelope_model_regular_graph_closed_form():
    # every vertex has degree d: pi_v = 1/V, p = 1-(1-1/V)^S, mean = B + V p, sigma^2 = V p (1-p)
    V, d, B, F = 50_000, 12, 256, (5, 3)
    mean, sigma = zg.envelope_model([d], [V], F, B)
    S0 = B * min(F[0], d)
    p0 = 1 - (1 - 1 / V) ** S0
    assert mean[0] == B and sigma[0] == 0
    assert abs(mean[1] - (B + V * p0)) < 1e-6 * mean[1]
    assert abs(sigma[1] - math.sqrt(V * p0 * (1 - p0))) < 1e-6 * sigma[1]
    S1 = S0 + (B + V * p0) * min(F[1], d)
    p1 = 1 - (1 - 1 / V) ** S1
    assert abs(mean[2] - (B + V * p1)) < 1e-6 * mean[2]
    # sparse regime: sigma^2 ~ mu, CV ~ 1/sqrt(mu)
    mu = V * p0
    assert abs(sigma[1] ** 2 / mu - 1) < 0.05


def test_envelope_model_against_simulation_of_its_own_assumptions():
    # Lemma 1's setting: S draws, each hitting vertex v with probability deg(v)/sum(deg); count distinct hits
    rnd = np.random.RandomState(0)
    deg = np.concatenate([np.full(4000, 2), np.full(800, 20), np.full(40, 400), np.zeros(500, dtype=int)])
    vals, cnts = np.unique(deg, return_counts=True)
    B, F = 64, (4,)
    mean, sigma = zg.envelope_model(vals.tolist(), cnts.tolist(), F, B, with_replacement=True)
    S = B * F[0] * (deg > 0).mean()  # seeds uniform over V, F draws when deg > 0
    pi = deg / deg.sum()
    sizes, sizes_poisson = [], []
    for _ in range(600):
        hits = rnd.choice(len(deg), size=int(round(S)), p=pi)
        sizes.append(len(np.unique(hits)))
        hits = rnd.choice(len(deg), size=rnd.poisson(S), p=pi)
        sizes_poisson.append(len(np.unique(hits)))
    assert abs((mean[1] - B) - np.mean(sizes)) < 0.02 * np.mean(sizes)
    # with exactly S draws the indicators are negatively correlated, so sum p(1-p) over-estimates the
    # spread (the conservative side); with a Poisson number of draws they are independent, as the proof assumes
    assert np.std(sizes) < 1.05 * sigma[1]
    assert abs(sigma[1] - np.std(sizes_poisson)) < 0.15 * sigma[1]


def _stats_graph():
    # 10_000 vertices: 9_000 of degree 3, 900 of degree 50, 100 of degree 1000
    return zg.Graph.from_degree_histogram([3, 50, 1000], [9000, 900, 100])


def test_plan_query_max_envelope_is_eq1_hop_by_hop():
    g = _stats_graph()
    info = g.plan_query((5, 4, 3), 100, zg.make_envelope(zg.ENV_MAX), feat_dim=16)
    assert list(info.node_cap[:4]) == [100, 600, 3000, 10_000]  # n(1+F), capped by |V|
    assert list(info.maxsg_nodes[:4]) == [100, 600, 3000, 10_000]
    assert list(info.edge_cap[:3]) == [500, 2400, 9000]
    assert info.envelope_bytes == info.maxsg_envelope_bytes
    assert info.workspace_bytes == info.envelope_bytes + info.scratch_bytes
    assert info.scratch_bytes >= 10_000 * 4 + 3 * 10_000 // 8  # id map, two hop bitmaps, the "seen" bitmap
    # hop-kernel launches: tickets for the rows of the previous frontier (tiles of 1024 / (lanes per row) = 128, 256, 256
    # rows) plus ranking tiles over the 313 bitmap words (a power of two of words each, about one pass of new rows per tile)
    assert list(info.grid_sample[:3]) == [1, 1 + 3, 3 + 10] and info.grid_compact == 10


def test_plan_query_model_envelope_uses_margin_and_z():
    g = _stats_graph()
    env = zg.make_envelope(zg.ENV_MODEL, margin=0.2, confidence=0.999, iterations=1000)
    info = g.plan_query((5, 4), 100, env, feat_dim=8)
    vals, cnts = g.degree_histogram()
    mean, sigma = zg.envelope_model(vals, cnts, (5, 4), 100)
    assert abs(info.z - 4.753) < 2e-3
    for h in (1, 2):
        want = math.ceil(max(1.2 * mean[h], mean[h] + info.z * sigma[h]))
        worst = min(10_000, info.node_cap[h - 1] * (1 + (5, 4)[h - 1]))
        assert info.node_cap[h] == max(info.node_cap[h - 1], min(worst, want))
        assert abs(info.model_mean[h] - mean[h]) < 1e-9
    assert info.envelope_bytes < info.maxsg_envelope_bytes
    # default margin is 20 %
    info2 = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_MODEL, confidence=0.999, iterations=1000), feat_dim=8)
    assert list(info2.node_cap[:3]) == list(info.node_cap[:3])


def test_plan_query_explicit_and_errors():
    g = _stats_graph()
    info = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_EXPLICIT, node_caps=[0, 450, 999_999]))
    assert list(info.node_cap[:3]) == [100, 450, 2250]  # second cap clamped to 450*(1+4)
    with pytest.raises(zg.ZgError):
        g.plan_query((5, 65), 100)
    with pytest.raises(zg.ZgError):
        g.plan_query((0,), 100)
    with pytest.raises(zg.ZgError):
        g.plan_query((5,), 20_000)
    with pytest.raises(zg.ZgError):
        g.plan_query((5,) * 9, 10)
    with pytest.raises(zg.ZgError) as ei:
        zg.Graph.from_degree_histogram([3, -1], [5, 5])
    assert ei.value.status == zg.EINVAL


def test_oracle_sizes_stay_inside_max_envelope_and_near_model(oracle):
    # realised sizes from the checker vs the planner's bounds, on a small R-MAT graph
    import torch
    from paper_2605_29346_amd import workloads as W
    g = W.rmat_graph(20_000, 400_000, 5)
    off = g.offsets.numpy()
    deg = np.diff(off)
    vals, cnts = np.unique(deg, return_counts=True)
    sg = zg.Graph.from_degree_histogram(vals.tolist(), cnts.tolist())
    fan, B = (10, 5), 256
    info = sg.plan_query(fan, B, zg.make_envelope(zg.ENV_MAX))
    og = oracle.Graph(off, g.indices.numpy())
    pool = W.SeedPool(g, B, 3)
    for s in range(5):
        b = og.sample_blocks(pool.batch_for(s).numpy(), fan, 100 + s)
        for h in range(3):
            assert b.n[h] <= info.node_cap[h]
        for h in range(2):
            assert b.E[h] <= info.edge_cap[h]
        assert b.n[2] < info.maxsg_nodes[2]  # shortfall + dedup keep it below the worst case


def test_plan_query_with_safe_twin_adds_the_worst_case_outputs_and_shares_the_scratch():
    g = _stats_graph()
    tight = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_MODEL), feat_dim=8)
    worst = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_MAX), feat_dim=8)
    both = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_MODEL, flags=zg.PLAN_SAFE_TWIN), feat_dim=8)
    assert tight.safe_envelope_bytes == 0
    assert both.envelope_bytes == tight.envelope_bytes and both.safe_envelope_bytes == worst.envelope_bytes
    assert both.scratch_bytes == worst.scratch_bytes  # one scratch region, sized for the twin
    assert both.workspace_bytes == tight.envelope_bytes + worst.envelope_bytes + worst.scratch_bytes
    assert list(both.node_cap[:3]) == list(tight.node_cap[:3])
    # the device-side fallback brings the same twin with it
    auto = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_MODEL, flags=zg.PLAN_AUTO_FALLBACK), feat_dim=8)
    assert (auto.safe_envelope_bytes, auto.workspace_bytes) == (both.safe_envelope_bytes, both.workspace_bytes)


def test_graph_aware_model_rejects_bad_arguments_before_touching_a_device():
    g = _stats_graph()
    L = zg.lib()
    mean = (ctypes.c_double * 9)()
    sigma = (ctypes.c_double * 9)()
    fan = (ctypes.c_int32 * 2)(5, 4)
    # a statistics-only handle has no edges to sweep
    assert L.zg_envelope_model_graph(g._h, fan, 2, 100, 0, None, 256, 10**9, None, mean, sigma) == zg.ESTATE
    assert L.zg_envelope_model_graph(None, fan, 2, 100, 0, None, 256, 10**9, None, mean, sigma) == zg.EINVAL
    assert L.zg_envelope_model_graph(g._h, fan, 2, 100, 0, None, None, 10**9, None, mean, sigma) == zg.EINVAL


def test_graph_mode_applies_the_lemma_cap_formula_to_the_callers_statistics():
    # ZG_ENV_GRAPH: caps = ceil(max((1 + margin) mean, mean + z sigma)) from the mean / sigma handed in (the output of
    # the graph-aware size model), clamped by the worst case and never below the previous hop's cap
    g = _stats_graph()
    mean, sigma = [0.0, 431.25, 1800.5], [0.0, 5.0, 400.0]
    env = zg.make_envelope(zg.ENV_GRAPH, margin=0.1, confidence=0.999, iterations=1000, model_mean=mean, model_sigma=sigma)
    info = g.plan_query((5, 4), 100, env, feat_dim=8)
    z = zg.normal_quantile(0.999 ** (1 / 1000))
    assert abs(info.z - z) < 1e-12
    assert info.node_cap[1] == math.ceil(1.1 * 431.25)                      # the margin term wins: 474.375 -> 475
    assert info.node_cap[2] == min(info.node_cap[1] * 5, math.ceil(1800.5 + z * 400.0))  # the z-sigma band wins
    assert [info.model_mean[h] for h in (1, 2)] == mean[1:] and [info.model_sigma[h] for h in (1, 2)] == sigma[1:]
    # defaults: margin 0.20, confidence 0.9999 over 1000 iterations
    info = g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_GRAPH, model_mean=mean, model_sigma=[0, 0, 0]), feat_dim=8)
    assert list(info.node_cap[1:3]) == [math.ceil(1.2 * 431.25), math.ceil(1.2 * 1800.5)]
    # a statistics-only handle is enough (the statistics are the caller's); nonsense is refused
    for bad in ([0.0, float("nan"), 1.0], [0.0, -3.0, 1.0], [0.0, float("inf"), 1.0]):
        with pytest.raises(zg.ZgError):
            g.plan_query((5, 4), 100, zg.make_envelope(zg.ENV_GRAPH, model_mean=bad, model_sigma=sigma))
    with pytest.raises(zg.ZgError):
        g.plan_query((5, 4), 100, zg.make_envelope(4))


def test_pilot_helper_adds_the_margin_to_the_largest_sizes():
    L = zg.lib()
    largest = (ctypes.c_int64 * 9)(999, 1000, 4321, 10)
    env = zg.Envelope()
    assert L.zg_envelope_from_pilot(largest, 3, 0.25, zg.PLAN_REPLACE, ctypes.byref(env)) == zg.OK
    assert env.mode == zg.ENV_EXPLICIT and env.flags == zg.PLAN_REPLACE
    assert list(env.node_caps[:4]) == [0, 1250, math.ceil(1.25 * 4321), 13]
    assert L.zg_envelope_from_pilot(largest, 3, -1.0, 0, ctypes.byref(env)) == zg.OK   # default margin 20 %
    assert list(env.node_caps[1:4]) == [1200, math.ceil(1.2 * 4321), 12]
    assert L.zg_envelope_from_pilot(largest, 0, 0.2, 0, ctypes.byref(env)) == zg.EINVAL
    assert L.zg_envelope_from_pilot(None, 3, 0.2, 0, ctypes.byref(env)) == zg.EINVAL
    largest[2] = -1
    assert L.zg_envelope_from_pilot(largest, 3, 0.2, 0, ctypes.byref(env)) == zg.EINVAL


def test_ticket_budget_is_an_envelope_field_not_an_environment_variable():
    g = _stats_graph()
    wide = g.plan_query((5, 4, 3), 2000, zg.make_envelope(zg.ENV_MAX))
    os.environ["ZG_MAX_TICKETS"] = "1"
    try:
        assert list(g.plan_query((5, 4, 3), 2000, zg.make_envelope(zg.ENV_MAX)).grid_sample[:3]) == list(wide.grid_sample[:3])
    finally:
        del os.environ["ZG_MAX_TICKETS"]
    narrow = g.plan_query((5, 4, 3), 2000, zg.make_envelope(zg.ENV_MAX, max_tickets=2))
    assert narrow.grid_sample[2] < wide.grid_sample[2] and list(narrow.node_cap[:4]) == list(wide.node_cap[:4])
    assert narrow.grid_sample[2] == 40 + 1  # 40 tickets of 256 old rows (a ticket holds 256 rows at most), one ranking tile
    assert narrow.grid_sample[0] == 8 and wide.grid_sample[0] == 16  # 2000 seeds: tiles of 128 rows, two per ticket (256 rows) when the budget asks


def test_the_binding_holds_none_of_the_envelope_arithmetic():
    # caps are computed behind the C ABI: the binding only forwards numbers
    src = open(os.path.join(ROOT, "paper_2605_29346_amd", "zg.py")).read()
    for token in ("max(", "ceil(", "sigma *", "* sigma", "1.0 + margin", "1 + margin"):
        assert token not in src, token


def test_every_device_flag_reaches_the_per_step_word():
    # a kernel that raises a ZG_FLAG_* bit in the sticky word raises it in the per-step word as well (that is what the
    # step log, the mailbox status and zg_step_status report): every atomicOr on `flags` is followed by its twin
    lines = open(os.path.join(ROOT, "paper_2605_29346_amd", "csrc", "zg_device.hip")).read().splitlines()
    sticky = [i for i, l in enumerate(lines) if "atomicOr(&" in l and "->flags," in l]
    assert len(sticky) >= 4
    for i in sticky:
        nxt = lines[i + 1]
        assert "->step_flags," in nxt and nxt.split("step_flags,")[1] == lines[i].split("flags,")[1], lines[i]


def test_build_id_names_the_sources_in_the_tree():
    from paper_2605_29346_amd import build as zg_build
    assert zg.lib().zg_build_id().decode() == zg_build.source_id()


def test_ranking_tiles_grow_to_16_words_per_lane_only_where_rows_not_the_budget_set_the_tile_count():
    # 100 M vertices of degree 12 (3.125 M bitmap words), 4096 seeds, explicit caps: the launch that ranks hop 0's
    # discoveries has rows for ~250 tickets, fewer than the budget allows: tiles of 16384 words (191 of them); the next
    # launch is at the ticket budget and the closing launch only ranks: tiles of 8192 words (382)
    g = zg.Graph.from_degree_histogram([12], [100_000_000])
    caps = [4096, 16_000, 120_000, 500_000]
    info = g.plan_query((15, 10, 5), 4096, zg.make_envelope(zg.ENV_EXPLICIT, node_caps=caps))
    words = 100_000_000 // 32
    t8, t16 = -(-words // 8192), -(-words // 16384)
    assert info.grid_sample[0] == 4096 // 64                      # fanout 15: 16 lanes per row, 64 rows per ticket
    assert info.grid_sample[1] == 4096 // 64 + t16                # fanout 10: 64 old rows per ticket + fat ranking tiles (255 tickets)
    assert info.grid_sample[2] == -(-16_000 // 256) + t8          # fanout 5: two tiles of 128 old rows per ticket, to stay in the budget
    assert info.grid_compact == t8
