"""Seeded random configurations within the documented limits, each run for a few iterations
against the oracle: sizes, block sizes (any multiple of 32, from one granule to 70 wave tiles),
partition counts up to one block per partition, densities from 1e-4 to 0.3, both comparators, all hyper-parameters, small capacities,
and a mix of plain and learning-rate-fused steps."""
import numpy as np
import pytest
import torch

from tests.parity import compare_step, log, make_pair

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _config(rng):
    n_g = int(rng.choice([rng.integers(1, 3000), rng.integers(3000, 70_000), rng.integers(70_000, 600_000)]))
    b = 32 * int(rng.choice([1, 2, 3, 8, 8, 16, 24, 31, 32, 33, 64, 100, 128, 256]))
    n_b = -(-n_g // b)
    P = int(min(n_b, rng.choice([1, 2, 3, 5, 8, 16, 33, 64, n_b])))
    P = max(1, min(P, 1024))
    d = float(rng.choice([1e-4, 1e-3, 0.01, 0.05, 0.3]))
    kw = dict(cmp_mode=int(rng.integers(0, 2)),
              alpha=float(rng.choice([1.0, 1.0, 1.2, 2.0])),
              beta=float(rng.choice([1.01, 1.1, 1.5])),
              gamma=float(rng.choice([0.0, 0.01, 0.05, 0.3])),
              blk_move=int(rng.choice([0, 1, 1, 2, 5])),
              min_blk=int(rng.choice([1, 1, 2, 4])),
              max_selected=int(rng.choice([0, 0, n_g, max(1, n_g // 50), 1])),
              want_err_norm=1)
    return n_g, b, P, d, kw


@pytest.mark.parametrize("seed", range(40))
def test_random_configuration(seed):
    rng = np.random.default_rng(1000 + seed)
    n_g, b, P, d, kw = _config(rng)
    scale = float(rng.choice([1e-3, 1.0, 50.0]))
    hot = int(rng.integers(0, n_g + 1)) if rng.random() < 0.6 else 0
    g0 = rng.laplace(0, scale, n_g).astype(np.float32)
    thr = float(np.quantile(np.abs(g0), 1.0 - d)) or scale
    log(f"case seed={seed} n_g={n_g} b={b} P={P} d={d} thr={thr:.4g} hot={hot} {kw}")
    x, o = make_pair(n_g, b, P, d, thr, **kw)
    for t in range(6):
        g = g0 if t == 0 else rng.laplace(0, scale, n_g).astype(np.float32)
        if hot:
            g = g.copy()
            g[:hot] *= 4.0                     # uneven load: Alg. 3 has something to move
        kind = int(rng.integers(0, 3))
        if kind == 0:
            x.step(torch.from_numpy(g).to(DEV))
            o.step(g)
        elif kind == 1:
            eta = float(np.float32(rng.choice([1.0, 0.3, -0.5])))
            x.step_scaled(torch.from_numpy(g).to(DEV), eta)
            o.step_scaled(g, 0, eta)
        else:
            eta = float(np.float32(rng.choice([1.0, 0.7])))
            gb = torch.from_numpy(g).to(DEV).to(torch.bfloat16)
            x.step_scaled(gb, eta)
            o.step_scaled(gb.view(torch.int16).cpu().numpy().view(np.uint16), 1, eta)
        compare_step(x, o, t, check_norm=True, tag=f"random-{seed}")
    x.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_configuration_with_many_tiles_per_block(seed):
    """Longer vectors with blocks of 4 to 70 wave tiles: blocks of whole segments (1 to 16 of
    them), and blocks that are not (1 to 16 counters each, generic sizes included); uneven load,
    small capacities, dense and sparse selections."""
    rng = np.random.default_rng(9000 + seed)
    b = int(rng.choice([4096, 8192, 12288, 16384, 20480, 65536, 4096 + 256, 8192 + 512, 16384 + 256,
                        32768 + 1024, 5120 + 32, 8224, 16352, 16416, 33056, 71648]))
    n_b = int(rng.integers(3, 40))
    n_g = int(b * (n_b - 1) + rng.integers(1, b + 1))
    P = int(min(n_b, rng.choice([1, 2, 3, 5, 8, n_b])))
    d = float(rng.choice([2e-4, 1e-3, 0.004, 0.02, 0.2]))
    kw = dict(cmp_mode=int(rng.integers(0, 2)), alpha=float(rng.choice([1.0, 1.2])),
              gamma=float(rng.choice([0.01, 0.05, 0.3])), blk_move=int(rng.choice([0, 1, 2])),
              min_blk=1, max_selected=int(rng.choice([0, 0, max(1, n_g // 500), n_g])), want_err_norm=1)
    hot = int(rng.integers(0, n_g + 1)) if rng.random() < 0.7 else 0
    g0 = rng.laplace(0, 1.0, n_g).astype(np.float32)
    thr = float(np.quantile(np.abs(g0), 1.0 - d))
    log(f"case tiles-per-block seed={seed} n_g={n_g} b={b} P={P} d={d} hot={hot} {kw}")
    x, o = make_pair(n_g, b, P, d, thr, **kw)
    for t in range(5):
        g = g0 if t == 0 else rng.laplace(0, 1.0, n_g).astype(np.float32)
        if hot:
            g = g.copy()
            g[:hot] *= 4.0
        x.step(torch.from_numpy(g).to(DEV))
        o.step(g)
        compare_step(x, o, t, check_norm=True, tag=f"tiles-per-block-{seed}")
    x.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_worker_view_configuration(seed):
    from tests.test_gpu_workers import _iteration, _make

    rng = np.random.default_rng(5000 + seed)
    n = int(rng.integers(2, 7))
    b = 32 * int(rng.choice([1, 3, 8, 16, 31, 32, 33, 64]))
    n_g = int(rng.integers(max(n * b, 2000), 200_000))
    d = float(rng.choice([1e-3, 0.01, 0.05]))
    kw = dict(cmp_mode=int(rng.integers(0, 2)), alpha=float(rng.choice([1.0, 1.5])),
              gamma=float(rng.choice([0.01, 0.1])), blk_move=int(rng.choice([0, 1, 3])),
              min_blk=int(rng.choice([1, 2])), max_selected=int(rng.choice([0, 0, max(1, n_g // 200)])),
              want_err_norm=1)
    hot = int(rng.integers(0, n_g // 2))
    g0 = rng.laplace(0, 1.0, n_g).astype(np.float32)
    thr = float(np.quantile(np.abs(g0), 1.0 - d))
    log(f"case workers seed={seed} n={n} n_g={n_g} b={b} d={d} hot={hot} {kw}")
    ctxs, w = _make(n_g, b, n, d, thr, **kw)
    for t in range(2 * n + 1):
        grads = []
        for i in range(n):
            g = rng.laplace(0, 1.0, n_g).astype(np.float32)
            g[:hot] *= 3.0
            grads.append(torch.from_numpy(g).to(DEV))
        _iteration(ctxs, w, grads, t, f"random-workers-{seed}", check_norm=True)
    for x in ctxs:
        x.close()
