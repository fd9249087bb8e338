"""GPU parity at the full sizes of the five configurations, in the launch configuration
the benchmark times, every output of every compared step checked element by element."""
import pytest
import torch

from paper_2402_13781_amd import synthetic
from tests.parity import log, make_pair, run_trajectory

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


# Steps and the stride of the compared ones.  Workload 4 is followed through the peak of its
# threshold transient (k' about 70 times k around iteration 25: the output overflows its
# capacity, only the first tiles emit, most tiles only count), its end (around iteration 50)
# and into the settled state; workload 5 far enough for the overflow and the count-only tiles;
# workload 3 through its dense segments.  Steps that are not compared still have their
# announced topology checked against the oracle's next Allocate.
@pytest.mark.timeout(900)
@pytest.mark.parametrize("index,steps,every", [(1, 20, 1), (2, 30, 3), (3, 21, 2), (4, 61, 10), (5, 7, 2)])
def test_full_size_configuration(index, steps, every):
    w = synthetic.WORKLOADS[index]
    log(f"case {w.name}: n_g={w.n_g} b={w.block_size} P={w.n_parts} d={w.density} steps={steps} every={every}")
    src = synthetic.GradientSource(w, DEV)
    g = src.grad(0)
    thr = synthetic.initial_threshold(g, w.density)
    x, o = make_pair(w.n_g, w.block_size, w.n_parts, w.density, thr)

    def grads():
        for t in range(steps):
            yield src.grad(t, out=g)

    run_trajectory(x, o, grads(), tag=w.name, every=every)
    x.close()
    del g, x
    torch.cuda.empty_cache()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("n_g,b,P,d,steps", [
    (20_000_000, 16384, 8, 2e-5, 4),     # a window of output ranks spans more tiles than fit LDS: spread by segment
    (80_000_000, 65536, 8, 4e-6, 4),     # ... and more segments than fit: every thread walks the levels itself
])
def test_sparse_selection_over_a_long_vector(n_g, b, P, d, steps):
    """Hundreds to thousands of wave tiles per selected gradient."""
    w = synthetic.WORKLOADS[5].scaled(n_g, b, P)
    log(f"case sparse: n_g={n_g} b={b} P={P} d={d}")
    src = synthetic.GradientSource(w, DEV)
    g = src.grad(0)
    thr = synthetic.initial_threshold(g, d)
    x, o = make_pair(n_g, b, P, d, thr, gamma=0.05)

    def grads():
        for t in range(steps):
            yield src.grad(t, out=g)

    run_trajectory(x, o, grads(), tag=f"sparse-{n_g}")
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
