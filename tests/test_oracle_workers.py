"""Pins for the n-worker oracle (Alg. 1 with per-worker gradients and residuals).

What fixes the expectations, none of it produced by the function under test:
* numpy written from the definitions: worker i's list is `flatnonzero(|acc_i| >= delta)`
  inside its own partition, the gathered list is the concatenation in rank order, every
  worker's values are `acc_i[idx_t]`, every worker zeroes at the whole gathered list;
* two special cases that reduce to the one-device oracle (itself pinned by brute force):
  n = 1, and n workers that all see the same gradient;
* Alg. 3's re-indexing of the partial-k vector against its cyclic allocation: the re-indexing must send worker i's count to the
  partition that `owner(t-1, i)` says it selected, and a hand-evaluated case.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2402_13781_amd import synthetic


def _grads(rng, n, n_g, scale=1e-3):
    return [rng.laplace(0.0, scale, n_g).astype(np.float32) for _ in range(n)]


def test_reindex_hand_case_and_owner_consistency():
    # n = 4, gathered after iteration t-1 = 1: worker i selected partition (1 + i) mod 4,
    # so [k0, k1, k2, k3] by rank is [k3, k0, k1, k2] by partition
    assert oracle.reindex([10, 20, 30, 40], 2).tolist() == [40, 10, 20, 30]
    assert oracle.reindex([10, 20, 30, 40], 1).tolist() == [10, 20, 30, 40]   # (t-1) mod n = 0
    assert oracle.reindex([10, 20, 30, 40], 5).tolist() == [10, 20, 30, 40]
    assert oracle.reindex([10, 20, 30, 40], 0).tolist() == [20, 30, 40, 10]   # (-1) mod 4 = 3
    for n in (1, 2, 3, 7):
        for t in range(1, 3 * n + 2):
            k_rank = np.arange(100, 100 + n, dtype=np.float64)
            k_part = oracle.reindex(k_rank, t)
            for i in range(n):
                assert k_part[oracle.owner(t - 1, i, n)] == k_rank[i]      # Alg. 3 (cyclic allocation)


def _check_workers_step(w, e_before, grads):
    """Everything that follows from Alg. 1 (the iteration body), given the oracle's own delta and topology."""
    n, n_g, b = w.n, w.n_g, w.b
    t = w.t - 1
    delta = w.threshold_used
    acc = [(e_before[i] + grads[i]).astype(np.float32) for i in range(n)]
    bp, pos = w.blk_part(0), w.blk_pos(0)
    assert pos[0] == 0 and np.array_equal(pos[1:], np.cumsum(bp)[:-1]) and bp.sum() == w.n_b
    lists, counts = [], []
    for i in range(n):
        p = (t % n + i) % n                                      # Alg. 3 (cyclic allocation)
        st, en = pos[p] * b, min((pos[p] + bp[p]) * b, n_g)
        own = st + np.flatnonzero(np.abs(acc[i][st:en]) >= delta)
        counts.append(own.size)
        lists.append(own[: w.cap])
    assert w.k_rank().tolist() == counts
    off = w.rank_off()
    assert off.tolist() == np.concatenate([[0], np.cumsum([len(l) for l in lists])]).tolist()
    idx_t = np.concatenate(lists).astype(np.uint32)
    assert np.array_equal(w.idx(), idx_t)
    assert w.k_actual == sum(counts)
    total = np.zeros(idx_t.size, np.float32)
    for i in range(n):
        want = acc[i][idx_t]                                     # value gather
        assert np.array_equal(w.values(i).view(np.uint32), want.view(np.uint32))
        total = want if i == 0 else (total + want).astype(np.float32)
        e_want = acc[i].copy()
        e_want[idx_t] = 0.0                                      # zeroing: the whole gathered list
        assert np.array_equal(w.residual(i).view(np.uint32), e_want.view(np.uint32))
    assert np.array_equal(w.sum().view(np.uint32), total.view(np.uint32))
    return counts


@pytest.mark.parametrize("n_g,b,n,d", [
    (8192, 256, 4, 0.01),
    (5000, 32, 3, 0.05),       # ragged tail
    (4096, 64, 7, 0.02),       # n does not divide n_b
])
def test_workers_step_matches_definitions(n_g, b, n, d):
    rng = np.random.default_rng(n_g + n)
    g0 = _grads(rng, n, n_g)
    thr = synthetic.initial_threshold(torch.from_numpy(g0[0]), d)
    w = oracle.Workers(n_g, b, n, d, thr, blk_move=1)
    e = [np.zeros(n_g, np.float32) for _ in range(n)]
    for t in range(3 * n + 2):                                   # every worker owns every partition
        g = g0 if t == 0 else _grads(rng, n, n_g)
        if t % 3 == 1:
            g[0][: n_g // 4] *= 6                                # skew the load so that Allocate moves
        w.step(g)
        _check_workers_step(w, e, g)
        e = [w.residual(i) for i in range(n)]


def test_next_allocate_uses_the_reindexed_counts():
    """The counts gathered by rank at iteration t drive iteration t+1's Allocate in partition order."""
    n_g, b, n = 8192, 128, 4
    rng = np.random.default_rng(3)
    w = oracle.Workers(n_g, b, n, 0.02, 2e-3, blk_move=1)
    for t in range(9):
        g = _grads(rng, n, n_g)
        for gi in g:
            gi[: n_g // 8] *= 20                                  # partition 0 is always overloaded
        bp_next, pos_next = w.blk_part(1).copy(), w.blk_pos(1).copy()
        k_rank = w.k_rank().astype(np.float64) if t else np.full(n, 0.02 * n_g / n)
        w.step(g)
        k_part = np.empty(n)
        for i in range(n):
            k_part[((t - 1) % n + i) % n] = k_rank[i]             # Python's % is the mathematical one
        _, want_bp, want_pos, _ = oracle.allocate(k_part, bp_next, pos_next, n_g, b, 1, 1, 1.0)
        assert np.array_equal(w.blk_part(0), want_bp) and np.array_equal(w.blk_pos(0), want_pos)
    assert w.blk_part(0)[0] < w.n_b // n                          # the hot partition has shrunk


def test_one_worker_is_the_one_device_oracle():
    n_g, b, d = 6000, 96, 0.03
    rng = np.random.default_rng(9)
    g0 = _grads(rng, 1, n_g)[0]
    thr = synthetic.initial_threshold(torch.from_numpy(g0), d)
    w = oracle.Workers(n_g, b, 1, d, thr)
    o = oracle.Oracle(n_g, b, 1, d, thr)
    for t in range(8):
        g = g0 if t == 0 else _grads(rng, 1, n_g)[0]
        w.step([g])
        o.step(g)
        assert np.array_equal(w.idx(), o.out_idx())
        assert np.array_equal(w.values(0).view(np.uint32), o.out_val().view(np.uint32))
        assert np.array_equal(w.residual(0).view(np.uint32), o.residual().view(np.uint32))
        assert w.threshold == o.threshold and w.k_actual == o.k_actual


def test_identical_gradients_reduce_to_the_one_device_oracle():
    """All workers see the same g: each selects its partition of the same acc, so the union is
    the one-device selection over all partitions, the topology and threshold follow the same
    trajectory, and every residual equals the one-device residual."""
    n_g, b, n, d = 20000, 160, 5, 0.01
    rng = np.random.default_rng(21)
    g0 = _grads(rng, 1, n_g)[0]
    g0[:3000] *= 8
    thr = synthetic.initial_threshold(torch.from_numpy(g0), d)
    w = oracle.Workers(n_g, b, n, d, thr, blk_move=2, max_selected=n_g)
    o = oracle.Oracle(n_g, b, n, d, thr, blk_move=2, max_selected=n_g)
    for t in range(12):
        g = g0 if t == 0 else _grads(rng, 1, n_g)[0]
        if t % 2:
            g[:3000] *= 8
        w.step([g] * n)
        o.step(g)
        order = np.argsort(w.idx(), kind="stable")
        assert np.array_equal(w.idx()[order], o.out_idx())
        for i in range(n):
            assert np.array_equal(w.values(i)[order].view(np.uint32), o.out_val().view(np.uint32))
            assert np.array_equal(w.residual(i).view(np.uint32), o.residual().view(np.uint32))
        assert np.array_equal(w.blk_part(0), o.blk_part(0)) and np.array_equal(w.blk_pos(0), o.blk_pos(0))
        # counts by rank, re-indexed by the partition each rank owned, are the per-partition counts
        pc = o.part_count()
        for i in range(n):
            assert w.k_rank()[i] == pc[(t % n + i) % n]
        assert w.threshold == o.threshold and w.k_actual == o.k_actual
        assert w.traffic_ratio() == o.traffic_ratio()
        assert abs(w.err_norm() - o.err_norm()) <= 1e-12 * max(o.err_norm(), 1e-30)


def test_a_worker_zeroes_entries_it_would_not_have_selected_itself():
    """Alg. 1 (zeroing of the sent entries) zeroes at the gathered list: an entry another worker selected is sent
    (with this worker's small value) and cleared here too."""
    n_g, b = 512, 128
    w = oracle.Workers(n_g, b, 2, 0.01, 1.0)
    ga = np.full(n_g, 0.25, np.float32)
    gb = np.full(n_g, -0.125, np.float32)
    ga[5] = 3.0          # partition 0, selected by worker 0 at t = 0
    gb[300] = -2.0       # partition 1, selected by worker 1 at t = 0
    ga[400] = 9.0        # partition 1 is not worker 0's at t = 0: stays in its residual
    w.step([ga, gb])
    assert w.idx().tolist() == [5, 300] and w.k_rank().tolist() == [1, 1]
    assert w.values(0).tolist() == [3.0, 0.25] and w.values(1).tolist() == [-0.125, -2.0]
    assert w.sum().tolist() == [2.875, -1.75]
    ea, eb = w.residual(0), w.residual(1)
    assert ea[5] == 0 and ea[300] == 0 and eb[5] == 0 and eb[300] == 0
    assert ea[400] == 9.0 and ea[0] == 0.25 and eb[0] == -0.125
    # next iteration the ownership rotates: worker 0 now owns partition 1 and sends index 400
    z = np.zeros(n_g, np.float32)
    w.step([z, z])
    assert 400 in w.idx().tolist() and w.residual(0)[400] == 0


def test_per_worker_capacity_keeps_the_rest_in_that_workers_residual():
    n_g, b, n = 2048, 128, 2
    rng = np.random.default_rng(2)
    g = [rng.normal(0, 1, n_g).astype(np.float32) for _ in range(n)]
    w = oracle.Workers(n_g, b, n, 0.5, 0.1, max_selected=50)
    w.step(g)
    assert w.cap == 50 and w.rank_off().tolist() == [0, 50, 100]
    own0 = np.flatnonzero(np.abs(g[0][:1024]) >= np.float32(0.1))
    assert w.k_rank()[0] == own0.size > 50                      # counts are untruncated
    assert np.array_equal(w.idx()[:50], own0[:50])
    e0 = w.residual(0)
    assert np.array_equal(e0[own0[50:]], g[0][own0[50:]])       # not sent: kept


def test_apply_update_equals_the_dense_update_with_zeros_elsewhere():
    """Alg. 1 (model update), x <- x - (1/n) g_t, where g_t is zero except at idx_t: the dense numpy
    expression and the sparse routine must agree bit for bit, and untouched entries stay."""
    rng = np.random.default_rng(4)
    n_g, n = 5000, 4
    x = rng.normal(0, 1, n_g).astype(np.float32)
    idx = rng.choice(n_g, 300, replace=False).astype(np.uint32)
    g = rng.normal(0, 3, 300).astype(np.float32)
    scale = np.float32(1.0 / n)
    dense = np.zeros(n_g, np.float32)
    dense[idx] = g
    want = (x - scale * dense).astype(np.float32)
    got = x.copy()
    oracle.apply_update(got, idx, g, scale)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    untouched = np.setdiff1d(np.arange(n_g), idx)
    assert np.array_equal(got[untouched].view(np.uint32), x[untouched].view(np.uint32))
    # scale 1 and g = x[idx]: the entries cancel exactly
    z = x.copy()
    oracle.apply_update(z, idx, x[idx], 1.0)
    assert not z[idx].any() and not np.signbit(z[idx]).any()


def test_apply_update_rounds_the_product_before_the_difference():
    scale, g, x0 = np.float32(1.4099537), np.float32(1.5942448), np.float32(1.3154374)
    fused = np.float32(float(x0) - float(scale) * float(g))      # what an FMA would round
    two_step = np.float32(x0 - np.float32(scale * g))
    assert fused != two_step
    x = np.full(8, x0, np.float32)
    oracle.apply_update(x, np.array([2, 5], np.uint32), np.array([g, g], np.float32), scale)
    assert x[2] == two_step and x[5] == two_step and x[0] == x0


def test_model_update_over_a_workers_iteration():
    """Lines 12 and 16 together on a small case: x - (1/n) * sum_i acc_i[idx_t], dense in numpy."""
    n_g, b, n = 2048, 128, 4
    rng = np.random.default_rng(8)
    grads = _grads(rng, n, n_g, 1.0)
    w = oracle.Workers(n_g, b, n, 0.02, 2.5)
    w.step(grads)
    idx = w.idx()
    assert idx.size > 0 and np.unique(idx).size == idx.size      # partitions are disjoint: no repeats
    total = np.zeros(n_g, np.float32)
    sent = np.zeros(n_g, bool)
    sent[idx] = True
    for i in range(n):                                             # rank-order sum of acc_i = g_i at t = 0
        total = np.where(sent, (total + grads[i]).astype(np.float32) if i else grads[i], 0).astype(np.float32)
    x0 = rng.normal(0, 1, n_g).astype(np.float32)
    want = (x0 - np.float32(1.0 / n) * total).astype(np.float32)
    x = x0.copy()
    oracle.apply_update(x, idx, w.sum(), 1.0 / n)
    assert np.array_equal(x.view(np.uint32), want.view(np.uint32))


def test_workers_threshold_uses_the_uncut_total():
    """Two workers, every gradient passes, capacity 10 per worker: k' = 512 (> beta * k = 281.6),
    not the 20 entries that were sent (< k / beta)."""
    n_g, b = 512, 128
    w = oracle.Workers(n_g, b, 2, 0.5, 0.5, gamma=0.01, beta=1.1, max_selected=10)
    g = [np.full(n_g, 1.0, np.float32), np.full(n_g, -2.0, np.float32)]
    w.step(g)
    assert w.k_rank().tolist() == [256, 256] and w.rank_off().tolist() == [0, 10, 20]
    assert w.k_actual == 512
    assert w.threshold == np.float32(np.float32(0.5) * np.float32(1.01))


def test_err_norm_per_worker_and_mean_against_numpy():
    """Eq. 1: the global error is the mean over the workers of the L2 norm of each worker's own
    residual.  Workers get gradients of different scales so that no two terms coincide and the
    mean differs from every term."""
    n_g, b, n = 6000, 96, 4
    rng = np.random.default_rng(123)
    w = oracle.Workers(n_g, b, n, 0.02, 2e-3)
    for t in range(3):
        grads = [rng.laplace(0.0, 1e-3 * (1 + 2 * i), n_g).astype(np.float32) for i in range(n)]
        w.step(grads)
        terms = [float(np.linalg.norm(w.residual(i).astype(np.float64))) for i in range(n)]
        assert len({round(v, 9) for v in terms}) == n
        for i in range(n):
            assert np.isclose(w.err_norm(i), terms[i], rtol=1e-12, atol=0.0)
        assert np.isclose(w.err_norm(), np.mean(terms), rtol=1e-12, atol=0.0)
        assert min(terms) < w.err_norm() < max(terms)


def test_workers_traffic_ratio_when_nothing_is_selected():
    """Eq. 5 at k' = 0 (0/0): reading taken is f(t) = 0, as in the one-device oracle."""
    n_g, n = 2048, 4
    w = oracle.Workers(n_g, 128, n, 0.1, 10.0)
    w.step([np.full(n_g, 0.5, np.float32) for _ in range(n)])
    assert w.k_actual == 0 and w.k_rank().tolist() == [0] * n
    assert w.traffic_ratio() == 0.0
    w.step([np.full(n_g, 20.0, np.float32) for _ in range(n)])   # every worker selects its whole partition
    assert w.k_actual == n_g and w.traffic_ratio() == 1.0
