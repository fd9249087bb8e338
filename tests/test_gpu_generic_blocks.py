"""Block sizes that are multiples of 32 but not of 256 (the granularity Alg. 2 (rounding of the block size) rounds
to): block and partition boundaries then fall inside the 256-gradient loads of a wavefront."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2402_13781_amd import binding, synthetic
from tests.parity import bits, log, make_pair, run_trajectory

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n_g,b,P,d", [
    (50_000 + 13, 32, 4, 0.01),         # eight blocks per wavefront load
    (100_003, 96, 7, 0.005),            # Alg. 2's own size for n_g = 1000, n_b = 10
    (300_000 + 1, 992, 5, 0.01),        # 31 x 32: just under a wave tile
    (400_000, 1056, 6, 0.02),           # 33 x 32: just over
    (70_000, 160, 3, 0.05),             # dense: tiles overflow their staging slots
    (9_000, 4512, 2, 0.01),             # larger than a workgroup's 4096, last block short
])
def test_generic_block_sizes_bit_exact(n_g, b, P, d):
    w = synthetic.WORKLOADS[5].scaled(n_g, b, P)       # skewed head: Alg. 3 moves boundaries
    src = synthetic.GradientSource(w, DEV)
    thr = synthetic.initial_threshold(src.grad(0), d)
    log(f"case generic n_g={n_g} b={b} P={P} d={d}")
    x, o = make_pair(n_g, b, P, d, thr, want_err_norm=1, blk_move=3)
    run_trajectory(x, o, (src.grad(t) for t in range(10)), tag=f"b={b}", check_norm=True)
    x.close()


# Blocks of many tiles that are not whole segments are counted by the streaming pass with
# several counters to a block (2, 4, 8, 16), which the control workgroup adds up; a tile inside
# one block adds once, a tile across a boundary lane by lane.
@pytest.mark.parametrize("b,P,d", [
    (5120, 7, 0.004),       # multiple of 256: counted per granule run, 2 counters per block
    (16640, 4, 0.01),       # 65 granules, 8 counters
    (8224, 5, 0.004),       # 257 x 32, 4 counters
    (16352, 3, 0.001),      # Alg. 2's own size for 138,357,544 gradients in 8445 blocks; 4 counters
    (16416, 4, 0.02),       # 513 x 32, 8 counters
    (33056, 2, 0.004),      # 1033 x 32, 16 counters
    (70000 - 70000 % 32, 2, 0.004),   # more than 64 tiles: 16 counters
])
def test_large_blocks_that_are_not_whole_segments(b, P, d):
    n_g = b * 11 + 5000 + 3
    w = synthetic.WORKLOADS[5].scaled(n_g, b, P)
    src = synthetic.GradientSource(w, DEV)
    thr = synthetic.initial_threshold(src.grad(0), d)
    log(f"case large generic n_g={n_g} b={b} P={P} d={d}")
    x, o = make_pair(n_g, b, P, d, thr, want_err_norm=1, blk_move=1)
    run_trajectory(x, o, (src.grad(t) for t in range(8)), tag=f"b={b}", check_norm=True)
    x.close()


def test_block_size_from_alg2_is_usable():
    """n_b = 100 blocks asked for, block size by Alg. 2 (block size) with the paper's multiple of 32."""
    n_g = 123_457
    b = binding.block_size_from_nb(n_g, 100, 32)
    assert b == oracle.block_size(n_g, 100) == 1216 and b % 256 != 0
    w = synthetic.WORKLOADS[1].scaled(n_g, b, 8)
    src = synthetic.GradientSource(w, DEV)
    thr = synthetic.initial_threshold(src.grad(0), 0.01)
    x, o = make_pair(n_g, b, 8, 0.01, thr)
    run_trajectory(x, o, (src.grad(t) for t in range(5)), tag="alg2-b")
    x.close()


# b = 416: boundaries inside wavefront loads; b = 8224 (257 x 32) and 12288 + 256: many tiles to a
# block with four counters each, partitions that start and end inside a wave tile
@pytest.mark.parametrize("b", [416, 8224, 12544])
def test_generic_blocks_scaled_16bit_and_worker_view(b):
    n_g, n, d = 150_000 + 7, 3, 0.01
    wl = synthetic.WORKLOADS[4].scaled(n_g, b, n)
    src = synthetic.GradientSource(wl, DEV)
    eta = 0.0625
    raw = lambda t: (src.grad(t) * 16.0).to(torch.bfloat16)
    thr = synthetic.initial_threshold(raw(0).float() * eta, d)
    # bf16 gradients with the learning rate fused in
    x, o = make_pair(n_g, b, n, d, thr)
    for t in range(5):
        g = raw(t)
        x.step_scaled(g, eta)
        o.step_scaled(g.view(torch.int16).cpu().numpy().view(np.uint16), 1, eta)
        assert np.array_equal(x.get_selected()[0].cpu().numpy().view(np.uint32), o.out_idx()), t
        assert np.array_equal(bits(x.residual.cpu().numpy()), bits(o.residual(copy=False))), t
        assert np.array_equal(x.get_block_counts(), o.block_count()), t
        assert np.float32(x.get_stats().delta_next) == o.threshold
    x.close()
    # worker view: the owned partition starts and ends inside wavefront loads
    cfg = binding.default_config(n_g=n_g, block_size=b, n_parts=n, density=d, threshold0=thr, blk_move=2)
    ctxs = [binding.ExDyna(cfg, DEV) for _ in range(n)]
    w = oracle.Workers(n_g, b, n, d, thr, blk_move=2)
    for t in range(7):
        grads = [src.grad(10 + t * n + i) for i in range(n)]
        for gi in grads:
            gi[:20_000] *= 5.0
        lists, counts = [], []
        for i, c in enumerate(ctxs):
            c.worker_select(grads[i], i)
            idx, val, _, ka, ke = c.get_selected()
            lists.append(idx.clone())
            counts.append(ka)
        stride = max(l.numel() for l in lists)
        idx_all = torch.full((n, stride), -1, dtype=torch.int32, device=DEV)
        for r, l in enumerate(lists):
            idx_all[r, :l.numel()] = l
        cd = torch.tensor(counts, dtype=torch.int64, device=DEV)
        vals = []
        for c in ctxs:
            v = torch.empty((n, stride), dtype=torch.float32, device=DEV)
            c.worker_exchange(idx_all, cd, v)
            vals.append(v)
        w.step([g.cpu().numpy() for g in grads])
        off = w.rank_off().astype(np.int64)
        assert counts == w.k_rank().tolist(), t
        for i, c in enumerate(ctxs):
            for r in range(n):
                assert np.array_equal(bits(vals[i][r, :lists[r].numel()].cpu().numpy()),
                                      bits(w.values(i)[off[r]:off[r + 1]])), (t, i, r)
            assert np.array_equal(bits(c.residual.cpu().numpy()), bits(w.residual(i, copy=False))), (t, i)
            assert np.float32(c.get_stats().delta_next) == w.threshold
            p = c.get_partitions(0)
            assert np.array_equal(p["blk_part"].astype(np.int64), w.blk_part(0)), t
            assert np.array_equal(p["blk_pos"].astype(np.int64), w.blk_pos(0)), t
        log(f"  [generic workers] t={t} k_i={counts} ok")
    for c in ctxs:
        c.close()
