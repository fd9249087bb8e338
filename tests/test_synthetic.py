"""The input generators: seeded, reproducible, shaped as the workload table says."""
import numpy as np
import torch

from paper_2402_13781_amd import synthetic


def test_workload_table_matches_the_configurations():
    w = synthetic.WORKLOADS
    assert [w[i].n_g for i in range(1, 6)] == [1_048_576, 11_689_512, 25_557_032, 138_357_544,
                                               1_500_000_000]
    assert [w[i].block_size for i in range(1, 6)] == [256, 4096, 4096, 16384, 65536]
    assert [w[i].n_parts for i in range(1, 6)] == [4, 8, 16, 32, 64]
    assert [w[i].density for i in range(1, 6)] == [0.01, 0.001, 0.01, 0.001, 0.0001]
    assert [w[i].iters for i in range(1, 6)] == [20, 100, 100, 200, 50]
    assert [w[i].n_blocks for i in range(1, 6)] == [4096, 2854, 6240, 8445, 22889]


def test_gradients_are_reproducible_and_step_dependent():
    for idx in range(1, 6):
        w = synthetic.WORKLOADS[idx].scaled(50_000)
        a = synthetic.GradientSource(w, "cpu").grad(3)
        b = synthetic.GradientSource(w, "cpu").grad(3)
        c = synthetic.GradientSource(w, "cpu").grad(4)
        assert a.dtype == torch.float32 and a.numel() == 50_000
        assert torch.equal(a, b) and not torch.equal(a, c)
        assert torch.isfinite(a).all()


def test_value_recipes():
    n = 400_000
    lap = synthetic.GradientSource(synthetic.WORKLOADS[1].scaled(n), "cpu").grad(0).double()
    assert abs(lap.abs().mean().item() - 1e-3) < 2e-5          # E|Laplace(0,s)| = s
    assert abs(lap.mean().item()) < 1e-5
    w5 = synthetic.WORKLOADS[5].scaled(n)
    g5 = synthetic.GradientSource(w5, "cpu").grad(0).double()
    head, rest = g5[: n // 20], g5[n // 20:]
    assert 15 < head.abs().mean().item() / rest.abs().mean().item() < 25   # x20 head
    w4 = synthetic.WORKLOADS[4].scaled(n)
    s4 = synthetic.GradientSource(w4, "cpu")
    first, last = s4.grad(0).abs().mean().item(), s4.grad(199).abs().mean().item()
    assert 80 < first / last < 125                                         # 1e-2 -> 1e-4
    w2 = synthetic.WORKLOADS[2].scaled(n)
    s2 = synthetic.GradientSource(w2, "cpu")
    assert int(s2.segment_sizes.sum()) == n and len(s2.segment_sizes) == 62
    assert (s2.segment_scales >= 1e-5).all() and (s2.segment_scales <= 1e-2).all()


def test_initial_threshold_is_the_order_statistic():
    g = torch.arange(1, 100_001, dtype=torch.float32) * 1e-5
    g[::2] *= -1
    thr = synthetic.initial_threshold(g, 0.01)
    sample = np.sort(np.abs(g.numpy()[::100]))
    assert thr == float(sample[int(np.ceil(0.99 * sample.size)) - 1])
