"""gcn_aggregate_static (the entry point that allocates nothing: its scratch memory is an array built into the library)
against gcn_aggregate, which runs the same kernels in a workspace of the caller's.  Run with -m gpu."""
import numpy as np
import pytest
import torch

from synth import rng, workloads
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2012_04930_amd import binding
    binding.lib()
    return binding


def _both(B, g, x, dtype):
    xd = torch.from_numpy(x).cuda()
    out = torch.full_like(xd, float("nan"))
    B.gcn_aggregate_static(g, xd, out, dtype=dtype)
    got = out.cpu().numpy()
    want = B.gcn_aggregate(g, xd, dtype=dtype).cpu().numpy()
    return got, want


def test_two_calls_in_a_row_the_second_on_a_smaller_input(B, oracle):
    """The array keeps what the last call left in it: a larger aggregation (dense tiles beside the gather, width 128)
    is followed by a smaller one (other graph, width 41, then bfloat16 rows), each compared with gcn_aggregate bit for
    bit (same kernels, same order of summation) and with the oracle to the stated tolerance."""
    big = workloads.reddit_partition(scale=0.085)            # 4.0 k vertices, community blocks: dense tiles in use
    small = workloads.chung_lu_mid(scale=0.03)               # 3,000 vertices, light and heavy rows, no tiles
    g_big, g_small = H.gpu_graph(B, big), H.gpu_graph(B, small)
    assert B.gcn_graph_tile_info(g_big)["in_use"]
    cases = [(g_big, big, 128, B.GCN_F32), (g_small, small, 41, B.GCN_F32), (g_small, small, 7, B.GCN_BF16),
             (g_big, big, 128, B.GCN_F32)]
    first = None
    for g, wl, width, dtype in cases:
        x = rng.normal_f32(width, 6, wl.n * width).reshape(wl.n, width)
        got, want = _both(B, g, x, dtype)
        np.testing.assert_array_equal(got, want)
        og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
        H.assert_close(got, oracle.aggregate(og, x), rtol=H.RTOL_BF16 if dtype == B.GCN_BF16 else H.RTOL_F32,
                       what="static scratch, width %d" % width)
        if first is None:
            first = got
    np.testing.assert_array_equal(got, first)                # the first case again, after the smaller ones


def test_limits_are_reported_not_exceeded(B):
    wl = workloads.chung_lu_mid(scale=0.3)                   # 30,000 vertices: width 256 needs 92 MB of scratch memory
    g = H.gpu_graph(B, wl)
    x = torch.zeros((wl.n, 256), device="cuda")
    out = torch.empty_like(x)
    with pytest.raises(B.GcnError) as e:
        B.gcn_aggregate_static(g, x, out)
    assert e.value.code == -4 and str(B.GCN_STATIC_SCRATCH_BYTES) in str(e.value)
    x = torch.ones((wl.n, 8), device="cuda")                 # 30,000 x 16 floats x 3 fits
    out = torch.empty_like(x)
    B.gcn_timing_enable(True)
    try:
        with pytest.raises(B.GcnError) as e:
            B.gcn_aggregate_static(g, x, out)
        assert e.value.code == -1
    finally:
        B.gcn_timing_enable(False)
    B.gcn_aggregate_static(g, x, out)
    np.testing.assert_array_equal(out.cpu().numpy(), B.gcn_aggregate(g, x).cpu().numpy())
