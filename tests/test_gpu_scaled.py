"""exdyna_step_scaled against the oracle: acc = fl(e + fl(eta * g)) with fp32, bf16 and
fp16 gradients (Alg. 1 (accumulate) with the learning rate inside the accumulate)."""
import numpy as np
import pytest
import torch

from paper_2402_13781_amd import binding, synthetic
from tests.parity import compare_step, log, make_pair

pytestmark = pytest.mark.gpu

DTYPES = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}


def _host_bits(g):
    """What the oracle takes: fp32 values, or the raw 16-bit patterns."""
    if g.dtype == torch.float32:
        return g.cpu().numpy()
    return g.view(torch.int16).cpu().numpy().view(np.uint16)


def _scaled_step(x, o, g, dt, eta):
    x.step_scaled(g, eta)
    o.step_scaled(_host_bits(g), dt, eta)


@pytest.mark.parametrize("dt", [0, 1, 2])
def test_scaled_trajectory(dt):
    # several workgroups, blocks that straddle wave tiles, ragged tail of 19 elements
    n, b, P, d = 700_000 + 19, 1536, 12, 0.003
    w = synthetic.WORKLOADS[4].scaled(n, b, P)
    src = synthetic.GradientSource(w, "cuda:0")
    eta = 0.0375                                     # not a power of two: the product rounds
    # unit-scale raw gradients so that fp16 keeps them out of its subnormal range
    raw = lambda t: (src.grad(t) * 1000.0).to(DTYPES[dt])
    g0 = raw(0)
    thr = synthetic.initial_threshold((g0.float() * eta), d)
    x, o = make_pair(n, b, P, d, thr, blk_move=2, want_err_norm=1)
    for t in range(10):
        g = raw(t)
        _scaled_step(x, o, g, dt, eta)
        ka, ke = compare_step(x, o, t, check_norm=True, tag=f"scaled dt={dt}")
        log(f"  [scaled dt={dt}] t={t} k'={ka} emitted={ke} ok")
    x.close()


def test_plain_and_scaled_steps_mix_on_one_context():
    n, b, P, d = 300_000 + 5, 1024, 8, 0.005
    w = synthetic.WORKLOADS[4].scaled(n, b, P)
    src = synthetic.GradientSource(w, "cuda:0")
    thr = synthetic.initial_threshold(src.grad(0), d)
    x, o = make_pair(n, b, P, d, thr)
    kinds = [None, 1, 0, None, 2, 1, None, 0, 2]     # odd count: both counter parities see each kind
    for t, dt in enumerate(kinds):
        g32 = src.grad(t)
        if dt is None:
            x.step(g32)
            o.step(g32.cpu().numpy())
        else:
            # eta * raw has the scale of g32, so the threshold stays in its working range
            eta = 1.0 / 768.0 if dt else 0.73
            raw = (g32 * 768.0).to(DTYPES[dt]) if dt else (g32 / 0.73)
            _scaled_step(x, o, raw, dt, eta)
        compare_step(x, o, t, tag=f"mix kind={dt}")
        log(f"  [mix] t={t} kind={dt} ok")
    x.close()


def test_scaled_special_values():
    """Infinities, signed zeros, the largest finite values and 16-bit subnormals widen exactly;
    a negative eta flips signs; eta = 0 keeps the residual.  (NaN gradients are left out: which
    payload a NaN product carries is not fixed by IEEE 754.)"""
    n, b, P = 4096 + 7, 256, 4
    for dt in (1, 2):
        x, o = make_pair(n, b, P, 0.01, 0.5, max_selected=n)
        pat = np.zeros(n, np.uint16)
        if dt == 2:
            specials = [0x7C00, 0xFC00, 0x8000, 0x0001, 0x83FF, 0x7BFF, 0xFBFF, 0x3C00, 0x0400]
        else:
            specials = [0x7F80, 0xFF80, 0x8000, 0x0001, 0x807F, 0x7F7F, 0xFF7F, 0x3F80, 0x0080]
        for j, v in enumerate(specials):
            pat[3 + 97 * j] = v
            pat[n - 1 - j] = v                          # in the ragged tail too
        g = torch.from_numpy(pat.view(np.int16)).to("cuda:0").view(DTYPES[dt])
        for t, eta in enumerate([1.0, -0.5, 0.0, 3.0e-5]):
            _scaled_step(x, o, g, dt, eta)
            compare_step(x, o, t, tag=f"special dt={dt} eta={eta}")
        x.close()
        log(f"  [special dt={dt}] ok")


def test_scaled_rejects_bad_arguments():
    n = 8192
    x = binding.ExDyna(binding.default_config(n_g=n, block_size=256, n_parts=2, density=0.01,
                                              threshold0=1.0), "cuda:0")
    g = torch.zeros(n, device="cuda:0")
    L = binding.load()
    import ctypes as C
    ptr = C.c_void_p(g.data_ptr())
    assert L.exdyna_step_scaled(x._h, ptr, 3, 1.0, None) == binding.EXDYNA_EINVAL
    assert L.exdyna_step_scaled(x._h, ptr, -1, 1.0, None) == binding.EXDYNA_EINVAL
    assert L.exdyna_step_scaled(x._h, ptr, 0, float("nan"), None) == binding.EXDYNA_EINVAL
    assert L.exdyna_step_scaled(x._h, ptr, 0, float("inf"), None) == binding.EXDYNA_EINVAL
    assert L.exdyna_step_scaled(x._h, None, 0, 1.0, None) == binding.EXDYNA_ENULL
    assert L.exdyna_step_scaled(None, ptr, 0, 1.0, None) == binding.EXDYNA_ENULL
    assert L.exdyna_step_scaled(x._h, C.c_void_p(g.data_ptr() + 4), 0, 1.0, None) == binding.EXDYNA_EALIGN
    assert x.get_stats().t == 0                         # nothing ran
    with pytest.raises(ValueError):
        x.step_scaled(g.double(), 1.0)
    x.close()
