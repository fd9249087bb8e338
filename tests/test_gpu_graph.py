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


def test_worker_view_iteration_after_graph_replays_owns_the_right_partition():
    """Alg. 3 (cyclic allocation) after HIP-graph replays: the replays advance the iteration counter
    on the device only, and the worker-view kernels take the owned partition from that counter.
    Every worker is given the same gradient, so whole steps and worker-view iterations are the
    same trajectory (Alg. 1 with identical workers) and a second, eager context supplies the lists
    the AllGather would deliver.  The worker's list, values, residual and threshold are compared
    with the n-worker oracle."""
    from oracle import oracle

    n, b, P, d, rank = 200_000 + 33, 1024, 4, 0.005, 1
    w = synthetic.WORKLOADS[5].scaled(n, b, P)
    src = synthetic.GradientSource(w, "cuda:0")
    thr = synthetic.initial_threshold(src.grad(0), d)
    x, _ = make_pair(n, b, P, d, thr)           # the worker: replayed graphs, then the worker view
    y, _ = make_pair(n, b, P, d, thr)           # plays the other workers' lists, always eager
    ow = oracle.Workers(n, b, P, d, thr)
    g_even = torch.empty(n, dtype=torch.float32, device="cuda:0")
    g_odd = torch.empty_like(g_even)

    def everyone_else(g):
        y.step(g)
        ow.step([g.cpu().numpy()] * P)

    t = 0
    for buf in (g_even, g_odd):
        buf.copy_(src.grad(t))
        x.step(buf)
        everyone_else(buf)
        t += 1
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        x.step(g_even)
        x.step(g_odd)
    for _ in range(2):                          # the device reaches t = 6; the host counted to 4
        g_even.copy_(src.grad(t))
        g_odd.copy_(src.grad(t + 1))
        graph.replay()
        everyone_else(g_even)
        everyone_else(g_odd)
        torch.cuda.synchronize()
        t += 2
    assert t == 6 and (t % P + rank) % P != (4 % P + rank) % P      # a stale counter would pick another partition

    g = src.grad(t)
    x.worker_select(g, rank)                    # no getter has run on x since the capture
    everyone_else(g)
    idx, val, off, ka, ke = y.get_selected()
    offs = off.cpu().numpy().astype(np.int64)
    assert ka == ke
    lens = np.diff(offs)
    stride = int(lens.max())
    idx_all = torch.full((P, stride), -1, dtype=torch.int32, device="cuda:0")
    counts = np.empty(P, np.int64)
    for r in range(P):
        p = oracle.owner(t, r, P)
        idx_all[r, :lens[p]] = idx[offs[p]:offs[p + 1]]
        counts[r] = lens[p]
    own_idx, own_val, _, oka, oke = x.get_selected()
    o_off = ow.rank_off().astype(np.int64)
    assert oka == oke == counts[rank] == ow.k_rank()[rank]
    assert np.array_equal(own_idx.cpu().numpy().view(np.uint32), ow.idx()[o_off[rank]:o_off[rank + 1]])
    assert np.array_equal(own_val.cpu().numpy().view(np.uint32),
                          ow.values(rank)[o_off[rank]:o_off[rank + 1]].view(np.uint32))
    val_all = torch.empty((P, stride), dtype=torch.float32, device="cuda:0")
    x.worker_exchange(idx_all, torch.from_numpy(counts).to("cuda:0"), val_all)
    torch.cuda.synchronize()
    assert np.array_equal(x.residual.cpu().numpy().view(np.uint32), ow.residual(rank, copy=False).view(np.uint32))
    s = x.get_stats()
    assert s.t == t + 1 == ow.t and np.float32(s.delta_next) == ow.threshold
    assert s.k_actual == ow.k_actual and s.bad_index == 0
    nxt = x.get_partitions(1)
    ow.step([src.grad(t + 1).cpu().numpy()] * P)
    assert np.array_equal(nxt["blk_part"].astype(np.int64), ow.blk_part(0))
    assert np.array_equal(nxt["blk_pos"].astype(np.int64), ow.blk_pos(0))
    log(f"  worker view after replays: t={t} own partition {(t % P + rank) % P} k_i={oka} ok")
    x.close()
    y.close()
