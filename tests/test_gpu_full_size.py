"""GPU parity at the full sizes of the five configurations, in the launch configuration
the benchmark times, every output of every compared step checked element by element."""
import pytest
import torch

from paper_2402_13781_amd import synthetic
from tests.parity import log, make_pair, run_trajectory

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.mark.timeout(900)
@pytest.mark.parametrize("index,steps", [(1, 20), (2, 12), (3, 6), (4, 4), (5, 2)])
def test_full_size_configuration(index, steps):
    w = synthetic.WORKLOADS[index]
    log(f"case {w.name}: n_g={w.n_g} b={w.block_size} P={w.n_parts} d={w.density} steps={steps}")
    src = synthetic.GradientSource(w, DEV)
    g = src.grad(0)
    thr = synthetic.initial_threshold(g, w.density)
    x, o = make_pair(w.n_g, w.block_size, w.n_parts, w.density, thr)

    def grads():
        for t in range(steps):
            yield src.grad(t, out=g)

    run_trajectory(x, o, grads(), tag=w.name)
    x.close()
    del g, x
    torch.cuda.empty_cache()
