"""exdyna_set_profiling / exdyna_get_kernel_ms: sampled per-kernel HIP events."""
import pytest
import torch

from paper_2402_13781_amd import binding

pytestmark = pytest.mark.gpu


def test_sampled_kernel_events():
    n = 1 << 20
    x = binding.ExDyna(binding.default_config(n_g=n, block_size=1024, n_parts=4, density=0.01,
                                              threshold0=2.0), "cuda:0")
    g = torch.randn(n, device="cuda:0")
    with pytest.raises(binding.ExDynaError):
        x.get_kernel_ms(0)                      # profiling is off
    with pytest.raises(binding.ExDynaError):
        x.set_profiling(4, 0)
    for _ in range(2):
        x.step(g)
    x.set_profiling(3, 4)                       # iterations 2, 6, 10, ... into a ring of 3
    for _ in range(13):
        x.step(g)                               # iterations 2..14: recorded 2, 6, 10, 14
    for t in (6, 10, 14):
        ms = x.get_kernel_ms(t)
        assert len(ms) == 2 and 0.0 < ms[0] < 50.0 and 0.0 < ms[1] < 50.0
    for t in (2, 7, 13, 15, 1):                 # overwritten, not sampled, not run, before profiling
        with pytest.raises(binding.ExDynaError) as ei:
            x.get_kernel_ms(t)
        assert ei.value.code == binding.EXDYNA_EINVAL
    x.set_profiling(0)
    x.step(g)
    assert x.get_stats().t == 16
    x.close()
