"""Checkpoint / resume: a context restored from saved state continues bit-identically."""
import numpy as np
import pytest
import torch

from paper_2402_13781_amd import binding, synthetic
from tests.parity import compare_step, log, make_pair

pytestmark = pytest.mark.gpu


def test_resume_continues_bit_exact():
    n, b, P, d = 500_000 + 19, 2048, 16, 0.004
    w = synthetic.WORKLOADS[5].scaled(n, b, P)
    src = synthetic.GradientSource(w, "cuda:0")
    thr = synthetic.initial_threshold(src.grad(0), d)
    x, o = make_pair(n, b, P, d, thr, blk_move=2, want_err_norm=1)
    for t in range(7):                       # odd number of steps: resume lands on the other parity
        g = src.grad(t)
        x.step(g)
        o.step(g.cpu().numpy())
        compare_step(x, o, t, check_norm=True, tag="before")
    state = x.get_state()
    saved_residual = x.residual.clone()
    assert len(state) == 40 + 2 * P * 4
    x.close()

    cfg = binding.default_config(n_g=n, block_size=b, n_parts=P, density=d, threshold0=123.0,
                                 blk_move=2, want_err_norm=1)
    y = binding.ExDyna(cfg, "cuda:0")
    y.set_state(state)
    y.residual.copy_(saved_residual)
    assert y.get_stats().t == 7
    assert y.get_state() == state            # round trip
    for t in range(7, 14):
        g = src.grad(t)
        y.step(g)
        o.step(g.cpu().numpy())
        compare_step(y, o, t, check_norm=True, tag="resumed")
        log(f"  resumed t={t} ok")

    # a state of another configuration, or a broken topology, is refused
    other = binding.ExDyna(binding.default_config(n_g=n, block_size=b, n_parts=P // 2, density=d,
                                                  threshold0=1.0), "cuda:0")
    with pytest.raises(binding.ExDynaError) as ei:
        other.set_state(state)
    assert ei.value.code == binding.EXDYNA_EINVAL
    bad = bytearray(state)
    bad[40] ^= 1                              # first partition size off by one
    with pytest.raises(binding.ExDynaError):
        y.set_state(bytes(bad))
    with pytest.raises(binding.ExDynaError):
        y.set_state(state[:-4])
    y.close()
    other.close()
