"""Context lifetime through the C ABI: a destroyed handle is refused, never read."""
import ctypes as C

import pytest
import torch

from paper_2402_13781_amd import binding

pytestmark = pytest.mark.gpu


def test_double_destroy_and_use_after_destroy_return_estate():
    L = binding.load()
    cfg = binding.default_config(n_g=10_000, block_size=256, n_parts=4, density=0.01, threshold0=1e-3)
    x = binding.ExDyna(cfg, "cuda:0")
    g = torch.zeros(10_000, dtype=torch.float32, device="cuda:0")
    x.step(g)
    torch.cuda.synchronize()
    h = C.c_void_p(x._h.value)
    assert L.exdyna_destroy(h) == binding.EXDYNA_OK
    x._h = C.c_void_p()                       # the wrapper must not destroy it again on its own
    assert L.exdyna_destroy(h) == binding.EXDYNA_ESTATE
    assert L.exdyna_step(h, C.c_void_p(g.data_ptr()), None) == binding.EXDYNA_ESTATE
    st = binding.Stats()
    assert L.exdyna_get_stats(h, C.byref(st)) == binding.EXDYNA_ESTATE
    assert L.exdyna_last_hip_error(h) == b""
    # a fresh context works, and the stale handle stays refused even if the allocator reuses the address
    y = binding.ExDyna(cfg, "cuda:0")
    y.step(g)
    assert y.get_stats().t == 1
    if y._h.value != h.value:
        assert L.exdyna_destroy(h) == binding.EXDYNA_ESTATE
    y.close()
