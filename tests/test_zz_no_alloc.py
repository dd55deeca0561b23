"""The entry point for callers that cannot allocate (zg_envelope_model_graph_static): its scratch is a static
device array of the library.  Through the C ABI, against zg_envelope_model_graph (caller-provided scratch), on
two calls in a row, the second on a smaller graph (the array keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_29346_amd import workloads as W
from paper_2605_29346_amd import zg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    zg.lib()


def _both(dg, fan, batch, replace, seed_prob=None):
    H = len(fan)
    mean, sigma = zg.graph_model(dg, fan, batch, with_replacement=replace, seed_prob=seed_prob)
    out = torch.full((2 * (H + 1),), -1.0, dtype=torch.float64, device="cuda")
    before = torch.cuda.memory_allocated()
    zg.graph_model_static(dg, fan, batch, out, with_replacement=replace, seed_prob=seed_prob)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    return np.array(mean), np.array(sigma), got[: H + 1], got[H + 1:]


def test_static_scratch_entry_point_matches_the_one_with_caller_scratch():
    big = W.rmat_graph(300_000, 4_000_000, 5)
    small = W.rmat_graph(7_001, 60_000, 6, offsets_dtype=torch.int32)
    for g, fan, batch, replace in ((big, (9, 6, 4), 500, False), (small, (5, 3), 64, True)):
        dg = zg.Graph(g.offsets.cuda(), g.indices.cuda())
        mean, sigma, smean, ssigma = _both(dg, fan, batch, replace)
        # the sums are integers (2^-32 fixed point) added in any order: the means are the same numbers; sigma goes
        # through one square root on either side (host libm, device) - equal to within an ulp or two
        assert np.array_equal(mean, smean), (mean, smean)
        assert np.allclose(sigma, ssigma, rtol=1e-14, atol=0), (sigma, ssigma)
        assert smean[0] == batch and ssigma[0] == 0 and np.all(smean[1:] > batch)
    # given seed probabilities, again on the small graph (third call, same array)
    prob = torch.zeros(7_001, device="cuda")
    prob[torch.arange(0, 7_001, 97, device="cuda")] = 1.0
    dg = zg.Graph(small.offsets.cuda(), small.indices.cuda())
    mean, sigma, smean, ssigma = _both(dg, (4, 4), 73, False, seed_prob=prob)
    assert np.array_equal(mean, smean) and np.allclose(sigma, ssigma, rtol=1e-14, atol=0)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    L = zg.lib()
    fan = (C.c_int32 * 2)(5, 4)
    out = torch.zeros(6, dtype=torch.float64, device="cuda")
    n = (1 << 20) + 1
    off = torch.zeros(n + 1, dtype=torch.int32, device="cuda")
    idx = torch.zeros(1, dtype=torch.int32, device="cuda")
    too_big = zg.Graph(off, idx[:0])
    assert L.zg_envelope_model_graph_static(too_big._h, fan, 2, 100, 0, None, None, out.data_ptr()) == zg.EINVAL
    assert b"ZG_STATIC_MODEL_MAX_NODES" in L.zg_last_error()
    stats = zg.Graph.from_degree_histogram([1, 2], [10, 10])
    assert L.zg_envelope_model_graph_static(stats._h, fan, 2, 4, 0, None, None, out.data_ptr()) == zg.ESTATE
    assert L.zg_envelope_model_graph_static(None, fan, 2, 4, 0, None, None, out.data_ptr()) == zg.EINVAL
    assert L.zg_envelope_model_graph_static(too_big._h, fan, 2, 100, 0, None, None, None) == zg.EINVAL
    assert float(out.abs().sum()) == 0.0
