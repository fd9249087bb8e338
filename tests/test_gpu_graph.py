"""A stream capture of two consecutive steps replays correctly (kernel nodes only, no memset)."""
import numpy as np
import pytest
import torch

from paper_2402_13781_amd import synthetic
from tests.parity import compare_step, log, make_pair

pytestmark = pytest.mark.gpu


def test_captured_pair_of_steps_replays_bit_exact():
    n, b, P, d = 300_000 + 77, 1024, 8, 0.005
    w = synthetic.WORKLOADS[5].scaled(n, b, P)
    src = synthetic.GradientSource(w, "cuda:0")
    thr = synthetic.initial_threshold(src.grad(0), d)
    x, o = make_pair(n, b, P, d, thr)
    g_even = torch.empty(n, dtype=torch.float32, device="cuda:0")
    g_odd = torch.empty_like(g_even)

    # two eager steps first (also warms up everything the capture must not initialise)
    t = 0
    for buf in (g_even, g_odd):
        buf.copy_(src.grad(t))
        x.step(buf)
        o.step(buf.cpu().numpy())
        compare_step(x, o, t, tag="eager")
        t += 1
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    g_even.copy_(src.grad(t))
    g_odd.copy_(src.grad(t + 1))
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        x.step(g_even)
        x.step(g_odd)
    # capture only records: the device state is still at iteration `t`
    assert x.get_stats().t == t
    for rep in range(4):
        g_even.copy_(src.grad(t))
        g_odd.copy_(src.grad(t + 1))
        graph.replay()
        torch.cuda.synchronize()
        # eager work and synchronisation between replays
        o.step(g_even.cpu().numpy())
        o.step(g_odd.cpu().numpy())
        t += 2
        # the library's host-side counter stayed at the captured pair; results are the device's
        idx, val, off, ka, ke = x.get_selected()
        assert ka == o.k_actual and ke == o.k_emitted
        assert np.array_equal(idx.cpu().numpy().view(np.uint32), o.out_idx())
        assert np.array_equal(val.cpu().numpy().view(np.uint32), o.out_val().view(np.uint32))
        assert np.array_equal(x.residual.cpu().numpy().view(np.uint32),
                              o.residual(copy=False).view(np.uint32))
        assert np.array_equal(x.get_block_counts(), o.block_count())
        parts = x.get_partitions(0)
        assert np.array_equal(parts["blk_part"].astype(np.int64), o.blk_part(0))
        assert np.array_equal(parts["blk_pos"].astype(np.int64), o.blk_pos(0))
        s = x.get_stats()
        assert s.t == t and np.float32(s.delta_next) == o.threshold
        log(f"  replay {rep}: t={t} k'={ka} ok")
    x.close()
