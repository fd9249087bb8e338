"""The ablations of the paper on synthetic inputs, through the trace tool: what rebalancing does to
the traffic ratio f(t) (Eq. 5, Sec. 5.3's comparison with static coarse partitions) and what
threshold scaling does to the density error (Eq. 6, Sec. 5.2).  Soft, directional checks of the
library's behaviour over a few hundred iterations; bit parity is checked elsewhere."""
import numpy as np
import pytest

from paper_2402_13781_amd import synthetic, trace
from tests.parity import log

pytestmark = pytest.mark.gpu


def test_rebalancing_lowers_the_traffic_ratio_on_a_skewed_workload():
    # 95 % of the selections fall into the first 5 % of the vector = inside partition 0 of 16
    w = synthetic.WORKLOADS[5].scaled(4_000_000, 4096, 16)
    tail = slice(200, 300)
    f = {}
    for name, kw in (("static", dict(static_partitions=True)), ("move1", dict(blk_move=1)),
                     ("move4", dict(blk_move=4))):
        rows = trace.run_trace(w, 300, **kw)
        f[name] = float(np.mean([r["traffic_ratio"] for r in rows[tail]]))
        if name == "static":
            assert all(r["moves"] == 0 for r in rows)
        log(f"  f(t) tail mean, {name}: {f[name]:.3f}")
    assert f["static"] > 15.5                  # everything in one of 16 partitions: f = P
    assert f["move1"] < 0.85 * f["static"]
    assert f["move4"] < 0.55 * f["static"]


def test_threshold_scaling_tracks_a_drifting_gradient_scale():
    # the gradient scale falls by 2.3 % per iteration; a fixed threshold first lets the error
    # feedback pile up far above the target density, then selects almost nothing
    w = synthetic.WORKLOADS[4].scaled(4_000_000, 4096, 16)
    scaled = trace.run_trace(w, 200)
    fixed = trace.run_trace(w, 200, fixed_threshold=True)
    assert len({r["delta_used"] for r in fixed}) == 1
    e_s = float(np.mean([r["density_error"] for r in scaled]))
    e_f = float(np.mean([r["density_error"] for r in fixed]))
    log(f"  mean density error: scaled {e_s:.4g}, fixed {e_f:.4g}")
    assert e_s < 0.5 * e_f
    # Alg. 5 moves the threshold by at most a factor (1 + gamma) per iteration
    d = np.array([r["delta_used"] for r in scaled], dtype=np.float64)
    ratio = d[1:] / d[:-1]
    assert ratio.max() <= 1.01 * (1 + 1e-6) and ratio.min() >= 0.99 * (1 - 1e-6)
