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


@pytest.mark.timeout(900)
def test_largest_gradient_vector_the_index_width_allows():
    """n_g = 2^32 - 1 (indices are 32 bits wide): 17 GB per vector, a ragged last wave tile that
    ends one short of 2^32, every index computation at the top of its range."""
    n_g = (1 << 32) - 1
    w = synthetic.WORKLOADS[5].scaled(n_g, 65536, 64)
    d = 1e-5
    log(f"case max-size: n_g={n_g} b=65536 P=64 d={d}")
    src = synthetic.GradientSource(w, DEV)
    g = src.grad(0)
    log("  gradient generated")
    thr = synthetic.initial_threshold(g, d)
    x, o = make_pair(n_g, 65536, 64, d, thr, blk_move=2, max_selected=8_000_000)
    # entries at the very end of the vector, inside the ragged tile, on both sides of the threshold
    g[n_g - 1] = 4.0 * thr
    g[n_g - 2] = -3.0 * thr
    g[n_g - 1024] = 2.0 * thr
    g[n_g - 3] = 0.6 * thr              # selected in the second iteration, once it has doubled
    run_trajectory(x, o, (g for _ in range(2)), tag="max-size")
    idx, _, _, ka, ke = x.get_selected()
    assert ka == ke                                  # nothing cut: the last pairs are the vector's last entries
    assert [int(i) & 0xFFFFFFFF for i in idx[-3:]] == [n_g - 3, n_g - 2, n_g - 1]
    x.close()
    del g, x
    torch.cuda.empty_cache()
