"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import json
import os
import re

import pytest

from paper_2402_13781_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _good(**kw):
    base = dict(n_g=1 << 20, block_size=256, n_parts=4, density=0.01, threshold0=1e-3)
    base.update(kw)
    return binding.default_config(**base)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "exdyna.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(exdyna_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(binding.SYMBOLS)
    L = binding.load()
    for name in declared:
        assert getattr(L, name) is not None


def test_default_config_values():
    c = binding.default_config()
    assert (c.alpha, c.beta, c.gamma, c.blk_move, c.min_blk, c.cmp_mode, c.max_selected,
            c.want_err_norm, c.reserved) == (1.0, 1.1, 0.01, 1, 1, 0, 0, 0, 0)
    assert binding.load().exdyna_default_config(None) == binding.EXDYNA_ENULL


def test_block_size_from_nb_matches_alg2_hand_cases(golden_dir):
    cases = json.load(open(os.path.join(golden_dir, "alg2_partition.json")))["block_size"]
    for c in cases:
        assert binding.block_size_from_nb(c["n_g"], c["n_b"], 32) == c["sz_blk"]
    assert binding.block_size_from_nb(138_357_544, 8445, 256) == 16383 - 16383 % 256
    with pytest.raises(binding.ExDynaError):
        binding.block_size_from_nb(100, 0, 32)


def test_workspace_bytes_accepts_the_five_configurations():
    from paper_2402_13781_amd.synthetic import WORKLOADS
    for w in WORKLOADS.values():
        cfg = _good(n_g=w.n_g, block_size=w.block_size, n_parts=w.n_parts, density=w.density)
        nbytes = binding.workspace_bytes(cfg)
        # staging slots dominate (8..64 pairs per 1024 gradients): below one fp32 vector
        assert w.n_g // 1024 * 16 * 8 <= nbytes < 2 * w.n_g * 4 + (64 << 20)


@pytest.mark.parametrize("bad", [
    dict(n_g=0), dict(n_g=1 << 32), dict(block_size=0), dict(block_size=48), dict(block_size=300),
    dict(n_parts=0), dict(n_parts=4097), dict(n_g=1 << 22, n_parts=1025), dict(density=0.0),
    dict(density=1.01), dict(density=float("nan")), dict(threshold0=0.0), dict(threshold0=-1.0),
    dict(threshold0=float("inf")), dict(threshold0=float("nan")), dict(cmp_mode=2),
    dict(alpha=0.99), dict(alpha=float("nan")), dict(beta=1.0), dict(gamma=-0.1), dict(gamma=1.0),
    dict(min_blk=0), dict(reserved=1), dict(max_selected=(1 << 20) + 1),
])
def test_bad_configurations_are_rejected(bad):
    with pytest.raises(binding.ExDynaError) as ei:
        binding.workspace_bytes(_good(**bad))
    assert ei.value.code == binding.EXDYNA_EINVAL


def test_init_and_step_argument_errors_without_a_gpu():
    L = binding.load()
    cfg = _good()
    h = C.c_void_p()
    need = binding.workspace_bytes(cfg)
    fake_res, fake_ws = C.c_void_p(0x7000_0000_1000), C.c_void_p(0x7000_1000_0000)
    assert L.exdyna_init(None, C.byref(cfg), fake_res, fake_ws, need, None) == binding.EXDYNA_ENULL
    assert L.exdyna_init(C.byref(h), None, fake_res, fake_ws, need, None) == binding.EXDYNA_ENULL
    assert L.exdyna_init(C.byref(h), C.byref(cfg), None, fake_ws, need, None) == binding.EXDYNA_ENULL
    assert L.exdyna_init(C.byref(h), C.byref(cfg), fake_res, None, need, None) == binding.EXDYNA_ENULL
    assert L.exdyna_init(C.byref(h), C.byref(_good(block_size=100)), fake_res, fake_ws, need,
                         None) == binding.EXDYNA_EINVAL
    assert L.exdyna_init(C.byref(h), C.byref(cfg), C.c_void_p(0x7000_0000_1004), fake_ws, need,
                         None) == binding.EXDYNA_EALIGN
    assert L.exdyna_init(C.byref(h), C.byref(cfg), fake_res, C.c_void_p(0x7000_1000_0010), need,
                         None) == binding.EXDYNA_EALIGN
    assert L.exdyna_init(C.byref(h), C.byref(cfg), fake_res, fake_ws, need - 1,
                         None) == binding.EXDYNA_ENOMEM
    assert not h.value
    assert L.exdyna_step(None, fake_res, None) == binding.EXDYNA_ENULL
    assert L.exdyna_step_scaled(None, fake_res, binding.EXDYNA_BF16, 1.0, None) == binding.EXDYNA_ENULL
    assert L.exdyna_worker_select(None, fake_res, binding.EXDYNA_F32, 1.0, 0, None) == binding.EXDYNA_ENULL
    assert L.exdyna_worker_exchange(None, fake_res, fake_res, 4, fake_res, None) == binding.EXDYNA_ENULL
    assert L.exdyna_get_stats(None, None) == binding.EXDYNA_ENULL
    assert L.exdyna_get_count_pointers(None, None, None) == binding.EXDYNA_ENULL
    assert L.exdyna_apply_update(None, fake_res, fake_res, fake_res, fake_res, 1, 4, 1.0, None) == binding.EXDYNA_ENULL
    assert L.exdyna_destroy(None) == binding.EXDYNA_ENULL
    assert L.exdyna_state_bytes(None, None) == binding.EXDYNA_ENULL
    assert L.exdyna_get_state(None, None, 0) == binding.EXDYNA_ENULL
    assert L.exdyna_set_state(None, None, 0, None) == binding.EXDYNA_ENULL
    # a block of host memory that is not a context
    junk = (C.c_uint64 * 256)()
    assert L.exdyna_step(C.cast(junk, C.c_void_p), fake_res, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_destroy(C.cast(junk, C.c_void_p)) == binding.EXDYNA_ESTATE


def test_a_handle_that_is_not_a_live_context_is_never_read():
    """Double destroy / use after destroy: the library looks a handle up in its table of live
    contexts before touching it.  An address in an unmapped page would fault if it were read."""
    L = binding.load()
    stale = C.c_void_p(0x10)
    fake = C.c_void_p(0x7000_0000_1000)
    st = binding.Stats()
    n = C.c_size_t()
    assert L.exdyna_destroy(stale) == binding.EXDYNA_ESTATE
    assert L.exdyna_destroy(stale) == binding.EXDYNA_ESTATE
    assert L.exdyna_step(stale, fake, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_step_scaled(stale, fake, binding.EXDYNA_F16, 1.0, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_worker_select(stale, fake, binding.EXDYNA_F32, 1.0, 0, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_worker_exchange(stale, fake, fake, 4, fake, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_get_stats(stale, C.byref(st)) == binding.EXDYNA_ESTATE
    assert L.exdyna_get_selected(stale, None, None, None, None, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_get_dims(stale, None, None) == binding.EXDYNA_ESTATE
    assert L.exdyna_state_bytes(stale, C.byref(n)) == binding.EXDYNA_ESTATE
    assert L.exdyna_set_profiling(stale, 4, 1) == binding.EXDYNA_ESTATE
    assert L.exdyna_last_hip_error(stale) == b""


def test_strerror_is_total():
    for code in range(-8, 2):
        assert binding.strerror(code)
