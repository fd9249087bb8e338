"""Worker view (exdyna_worker_select / exdyna_worker_exchange) against the n-worker oracle:
one context per worker on the one GPU, the test plays the two collectives of Alg. 1."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2402_13781_amd import binding, synthetic
from tests.parity import bits, log

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _make(n_g, b, n, d, thr, **kw):
    cfg = binding.default_config(n_g=n_g, block_size=b, n_parts=n, density=d, threshold0=thr, **kw)
    ctxs = [binding.ExDyna(cfg, DEV) for _ in range(n)]
    w = oracle.Workers(n_g, b, n, d, thr, alpha=cfg.alpha, beta=cfg.beta, gamma=cfg.gamma,
                       blk_move=cfg.blk_move, min_blk=cfg.min_blk, cmp_mode=cfg.cmp_mode,
                       max_selected=cfg.max_selected)
    assert all(x.capacity == w.cap for x in ctxs)
    return ctxs, w


def _iteration(ctxs, w, grads, t, tag, check_norm=False):
    """select on every worker, AllGather by hand, exchange on every worker, compare everything."""
    n = len(ctxs)
    lists, counts = [], []
    for i, x in enumerate(ctxs):
        x.worker_select(grads[i], i)
        idx, val, off, ka, ke = x.get_selected()
        lists.append((idx.clone(), val.clone(), ke))
        counts.append(ka)
    stride = max(ke for _, _, ke in lists)
    # rows padded with an index that must never be dereferenced
    idx_all = torch.full((n, stride), -1, dtype=torch.int32, device=DEV)
    for r, (idx, _, ke) in enumerate(lists):
        idx_all[r, :ke] = idx
    # the counts as a collective would see them: straight from device memory
    counts_dev = torch.cat([x.count_tensors()[0] for x in ctxs]).contiguous()
    assert counts_dev.tolist() == counts
    assert [int(x.count_tensors()[1]) for x in ctxs] == [ke for _, _, ke in lists]
    vals = []
    for x in ctxs:
        val_all = torch.full((n, stride), float("nan"), dtype=torch.float32, device=DEV)
        x.worker_exchange(idx_all, counts_dev, val_all)
        vals.append(val_all)
    torch.cuda.synchronize()

    w.step([g.cpu().numpy() for g in grads])
    where = f"{tag} t={t}"
    assert counts == w.k_rank().tolist(), where
    off = w.rank_off().astype(np.int64)
    o_idx = w.idx()
    for r, (idx, val, ke) in enumerate(lists):
        assert ke == off[r + 1] - off[r], where
        assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx[off[r]:off[r + 1]]), where
    for i, x in enumerate(ctxs):
        got = vals[i].cpu().numpy()
        want = w.values(i)
        for r in range(n):
            ke = lists[r][2]
            assert np.array_equal(bits(got[r, :ke]), bits(want[off[r]:off[r + 1]])), (where, i, r)
            assert not got[r, ke:].any() and not np.isnan(got[r, ke:]).any(), (where, i, r)   # padding is 0
        # the worker's own values are also what its list reported
        assert np.array_equal(bits(lists[i][1].cpu().numpy()), bits(want[off[i]:off[i + 1]])), where
        assert np.array_equal(bits(x.residual.cpu().numpy()), bits(w.residual(i, copy=False))), (where, i)
        s = x.get_stats()
        assert s.t == t + 1 == w.t
        assert np.float32(s.delta_used) == w.threshold_used and np.float32(s.delta_next) == w.threshold, where
        assert s.k_actual == w.k_actual and s.k_emitted == off[-1], where
        assert s.k_max_part == max(counts) and s.bad_index == 0
        assert s.traffic_ratio == w.traffic_ratio(), where
        assert s.padding_overhead == oracle.padding_overhead(counts), where
        assert s.overflow == int(any(c > x.capacity for c in counts))
        used, nxt = x.get_partitions(0), x.get_partitions(1)
        assert np.array_equal(used["blk_part"].astype(np.int64), w.blk_part(0)), where
        assert np.array_equal(used["blk_pos"].astype(np.int64), w.blk_pos(0)), where
        # the next topology is what the oracle's next Allocate will produce: checked one step later
        x._announced = nxt
        pc = x.get_part_counts()
        for r in range(n):
            assert pc[(t % n + r) % n] == counts[r], where         # Alg. 3 (re-indexing of the partial-k vector)
        if check_norm:
            want_n = w.err_norm(i)
            assert abs(s.err_norm - want_n) <= 1e-5 * max(want_n, 1e-30), (where, s.err_norm, want_n)
    # the reduced values: sum of the workers' buffers in rank order = the oracle's g_t
    total = vals[0].clone()
    for v in vals[1:]:
        total += v
    got_sum = np.concatenate([total[r, :lists[r][2]].cpu().numpy() for r in range(n)]) if stride else np.empty(0, np.float32)
    assert np.array_equal(bits(got_sum), bits(w.sum())), where
    return counts


def _run(n_g, b, n, d, steps, tag, hot=None, check_norm=False, **kw):
    wl = synthetic.WORKLOADS[4].scaled(n_g, b, n)
    src = synthetic.GradientSource(wl, DEV)

    def grad(t, i):
        g = src.grad(t * n + i)
        if hot:
            g[: hot[0]] *= hot[1]
        return g

    thr = synthetic.initial_threshold(grad(0, 0), d)
    ctxs, w = _make(n_g, b, n, d, thr, want_err_norm=int(check_norm), **kw)
    prev = None
    for t in range(steps):
        grads = [grad(t, i) for i in range(n)]
        counts = _iteration(ctxs, w, grads, t, tag, check_norm=check_norm)
        if prev is not None:
            for p in prev:
                assert np.array_equal(p["blk_part"].astype(np.int64), w.blk_part(0)), (tag, t)
                assert np.array_equal(p["blk_pos"].astype(np.int64), w.blk_pos(0)), (tag, t)
        prev = [x._announced for x in ctxs]
        log(f"  [{tag}] t={t} k_i={counts} delta_next={float(w.threshold):.6g} ok")
    moved = not np.array_equal(w.blk_part(0), oracle.partition(w.n_b, n)[0])
    for x in ctxs:
        x.close()
    return moved


def test_workers_basic():
    # ragged tail; blocks are whole wave tiles
    _run(300_000 + 19, 1024, 4, 0.004, 9, "workers n=4", check_norm=True)


def test_workers_boundaries_inside_wave_tiles_and_rebalancing():
    # b = 768: partition boundaries fall inside wave tiles; the hot head makes Alg. 3 move them
    moved = _run(250_000 + 777, 768, 3, 0.01, 10, "workers b=768", hot=(40_000, 6.0), blk_move=2,
                 check_norm=True)
    assert moved


def test_workers_dense_tiles_and_capacity():
    # d = 0.05: many tiles select more than their staging slots hold (re-read path, also on
    # partition boundaries); a small capacity cuts every worker's list
    _run(120_000 + 5, 256, 5, 0.05, 7, "workers dense", max_selected=700)


def test_workers_at_the_full_size_of_a_configuration():
    # cfg 2 as it stands (n_g = 11,689,512, b = 4096, 8 workers), each worker its own gradient
    wl = synthetic.WORKLOADS[2]
    src = synthetic.GradientSource(wl, DEV)
    n = wl.n_parts
    thr = synthetic.initial_threshold(src.grad(0), wl.density)
    ctxs, w = _make(wl.n_g, wl.block_size, n, wl.density, thr)
    for t in range(3):
        grads = [src.grad(t * n + i) for i in range(n)]
        counts = _iteration(ctxs, w, grads, t, "workers cfg2")
        log(f"  [workers cfg2] t={t} k_i={counts} ok")
    for x in ctxs:
        x.close()


def test_one_worker_view_equals_the_whole_step():
    n_g, b, d = 200_000 + 3, 512, 0.005
    wl = synthetic.WORKLOADS[4].scaled(n_g, b, 1)
    src = synthetic.GradientSource(wl, DEV)
    thr = synthetic.initial_threshold(src.grad(0), d)
    cfg = binding.default_config(n_g=n_g, block_size=b, n_parts=1, density=d, threshold0=thr)
    a, x = binding.ExDyna(cfg, DEV), binding.ExDyna(cfg, DEV)
    for t in range(5):
        g = src.grad(t)
        a.step(g)
        x.worker_select(g, 0)
        idx, val, off, ka, ke = x.get_selected()
        x.worker_exchange(idx.view(1, -1).contiguous(), torch.tensor([ka], dtype=torch.int64, device=DEV),
                          torch.empty((1, ke), dtype=torch.float32, device=DEV))
        ia, va, _, kaa, kea = a.get_selected()
        assert (ka, ke) == (kaa, kea) and torch.equal(idx, ia) and torch.equal(val.view(torch.int32), va.view(torch.int32))
        assert torch.equal(a.residual.view(torch.int32), x.residual.view(torch.int32))
        assert a.get_stats().delta_next == x.get_stats().delta_next
    a.close()
    x.close()


def test_worker_view_state_machine_and_bad_input():
    n_g, b, n = 50_000, 256, 2
    cfg = binding.default_config(n_g=n_g, block_size=b, n_parts=n, density=0.01, threshold0=0.5)
    x = binding.ExDyna(cfg, DEV)
    L = binding.load()
    g = torch.zeros(n_g, device=DEV)
    g[10] = 2.0            # partition 0: worker 0's at t = 0
    g[40_000] = -3.0       # partition 1: not selected by worker 0, but gathered from "worker 1"
    gp = C.c_void_p(g.data_ptr())
    counts = torch.tensor([1, 2], dtype=torch.int64, device=DEV)
    idx_all = torch.tensor([[10, 0], [40_000, n_g + 5]], dtype=torch.int32, device=DEV)
    val_all = torch.zeros((2, 2), dtype=torch.float32, device=DEV)
    ex = lambda: L.exdyna_worker_exchange(x._h, C.c_void_p(idx_all.data_ptr()), C.c_void_p(counts.data_ptr()),
                                          2, C.c_void_p(val_all.data_ptr()), None)
    assert ex() == binding.EXDYNA_ESTATE                                   # nothing selected yet
    assert L.exdyna_worker_select(x._h, gp, 0, 1.0, 2, None) == binding.EXDYNA_EINVAL      # rank >= P
    assert L.exdyna_worker_select(x._h, gp, 5, 1.0, 0, None) == binding.EXDYNA_EINVAL
    assert L.exdyna_worker_select(x._h, gp, 0, float("inf"), 0, None) == binding.EXDYNA_EINVAL
    assert L.exdyna_worker_select(None, gp, 0, 1.0, 0, None) == binding.EXDYNA_ENULL
    x.worker_select(g, 0)
    assert L.exdyna_step(x._h, gp, None) == binding.EXDYNA_ESTATE          # exchange pending
    assert L.exdyna_worker_select(x._h, gp, 0, 1.0, 0, None) == binding.EXDYNA_ESTATE
    with pytest.raises(binding.ExDynaError):
        x.get_state()
    idx, val, off, ka, ke = x.get_selected()
    assert (ka, ke) == (1, 1) and idx.tolist() == [10] and val.tolist() == [2.0]
    assert L.exdyna_worker_exchange(x._h, None, C.c_void_p(counts.data_ptr()), 2, None, None) == binding.EXDYNA_ENULL
    assert L.exdyna_worker_exchange(x._h, C.c_void_p(idx_all.data_ptr()), None, 2,
                                    C.c_void_p(val_all.data_ptr()), None) == binding.EXDYNA_ENULL
    assert ex() == binding.EXDYNA_OK
    s = x.get_stats()
    assert s.t == 1 and s.bad_index == 1 and s.k_actual == 3             # the index beyond n_g was skipped
    assert val_all.tolist() == [[2.0, 0.0], [-3.0, 0.0]]
    r = x.residual
    assert r[10] == 0 and r[40_000] == 0 and float(r.abs().sum()) == 0.0
    assert ex() == binding.EXDYNA_ESTATE
    x.step(g)                                                              # whole-step calls work again
    assert x.get_stats().t == 2
    x.close()
