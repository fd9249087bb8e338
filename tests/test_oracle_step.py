"""Pins for the oracle's whole-step state machine (Alg. 1 (the iteration body), Alg. 4).

The expectations are what the paper's definitions reduce to in numpy: the
selected set is `flatnonzero(|acc| >= delta)` (Alg. 4's `where`), its size is
the position of delta in the fully sorted magnitudes, the sent values plus the
new residual reassemble acc exactly, partitions tile the vector.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2402_13781_amd import synthetic


def _rand_grad(rng, n, scale=1e-3):
    return (rng.laplace(0.0, scale, n)).astype(np.float32)


def _check_step(o, e_before, g, cmp_mode=0):
    """All per-step facts that follow from the definitions, given the oracle's own delta/topology."""
    acc = (e_before + g).astype(np.float32)                 # one fp32 add (Alg. 1 (accumulate))
    delta = o.threshold_used
    mag = np.abs(acc)
    mask = mag > delta if cmp_mode else mag >= delta
    want_idx = np.flatnonzero(mask).astype(np.uint32)       # Alg. 4: where(...)
    # brute force through a full sort: count = #sorted magnitudes at/above delta
    srt = np.sort(mag[~np.isnan(mag)])
    side = "right" if cmp_mode else "left"
    assert o.k_actual == srt.size - np.searchsorted(srt, delta, side=side)
    assert o.k_actual == want_idx.size

    bp, pos = o.blk_part(0), o.blk_pos(0)
    # partitions: contiguous, non-overlapping, cover all n_g (Sec. 4.1)
    assert pos[0] == 0 and np.array_equal(pos[1:], np.cumsum(bp)[:-1]) and bp.sum() == o.n_b
    st = pos * o.b
    en = np.minimum((pos + bp) * o.b, o.n_g)
    pc = o.part_count()
    for p in range(o.P):
        assert pc[p] == np.count_nonzero(mask[st[p]:en[p]])
    assert pc.sum() == o.k_actual

    ke = o.k_emitted
    assert ke == min(o.k_actual, o.cap)
    idx, val = o.out_idx(), o.out_val()
    assert np.array_equal(idx, want_idx[:ke])               # ascending, global index order
    assert np.array_equal(val.view(np.uint32), acc[idx].view(np.uint32))   # values = acc[idx]
    off = o.part_off()
    assert off[0] == 0 and off[-1] == ke
    assert np.array_equal(off[1:], np.minimum(np.cumsum(pc), o.cap))

    # block counts
    bc = o.block_count()
    pad = np.zeros(o.n_b * o.b, bool)
    pad[: o.n_g] = mask
    assert np.array_equal(bc, pad.reshape(o.n_b, o.b).sum(1).astype(np.uint32))

    # error feedback: sent + residual == acc, exactly (Alg. 1 (zeroing and residual carry))
    e_after = o.residual()
    sent = np.zeros_like(acc)
    sent[idx] = val
    want_e = acc.copy()
    want_e[idx] = 0.0
    assert np.array_equal(e_after.view(np.uint32), want_e.view(np.uint32))
    recon = np.where(np.isin(np.arange(o.n_g), idx), sent, e_after)
    assert np.array_equal(recon.view(np.uint32), acc.view(np.uint32))
    assert not np.any(np.signbit(e_after[idx]))             # selected slots hold +0
    return acc


@pytest.mark.parametrize("n_g,b,P,d", [
    (4096, 256, 4, 0.01),
    (4000, 32, 5, 0.05),       # ragged tail, block of one warp's width
    (1000, 96, 3, 0.1),        # Alg. 2's own 32-multiple block size for n_g=1000, n_b=10
    (257, 256, 2, 0.2),        # last block holds a single element
    (8192, 8192, 1, 0.01),     # one partition, one block: plain hard-threshold selection
])
def test_step_matches_definitions(n_g, b, P, d):
    rng = np.random.default_rng(n_g + P)
    g0 = _rand_grad(rng, n_g)
    thr = synthetic.initial_threshold(torch.from_numpy(g0), d)
    o = oracle.Oracle(n_g, b, P, d, thr)
    e = np.zeros(n_g, np.float32)
    for t in range(12):
        g = g0 if t == 0 else _rand_grad(rng, n_g)
        assert o.t == t
        o.step(g)
        _check_step(o, e, g)
        e = o.residual()


def test_tie_is_selected_by_ge_and_not_by_gt():
    n = 512
    g = np.full(n, 0.25, np.float32)
    g[7] = -0.5         # exactly at the threshold, negative sign
    g[300] = 0.5        # exactly at the threshold
    g[301] = np.nextafter(np.float32(0.5), np.float32(0))   # one ulp below
    g[302] = np.nextafter(np.float32(0.5), np.float32(1))   # one ulp above
    o = oracle.Oracle(n, 256, 2, 0.01, 0.5, cmp_mode=0)
    o.step(g)
    assert o.out_idx().tolist() == [7, 300, 302]
    o = oracle.Oracle(n, 256, 2, 0.01, 0.5, cmp_mode=1)
    o.step(g)
    assert o.out_idx().tolist() == [302]


def test_nan_inf_negative_zero():
    n = 256
    g = np.zeros(n, np.float32)
    g[3] = np.nan
    g[4] = np.inf
    g[5] = -np.inf
    g[6] = -0.0
    g[7] = -2.0
    o = oracle.Oracle(n, 64, 2, 0.1, 1.0)
    o.step(g)
    assert o.out_idx().tolist() == [4, 5, 7]                # NaN never compares true
    assert o.out_val().tolist() == [np.inf, -np.inf, -2.0]
    e = o.residual()
    assert np.isnan(e[3]) and e[4] == 0 and e[5] == 0 and e[7] == 0
    assert not np.signbit(e[5]) and not np.signbit(e[7])    # +0 where sent
    assert e[6] == 0 and not np.signbit(e[6])               # IEEE: (+0) + (-0) = +0


def test_error_feedback_accumulates_until_selected():
    """Sec. 2: an unselected gradient is kept and gets its chance once the sum is large enough."""
    n = 64
    g = np.zeros(n, np.float32)
    g[10] = 0.3
    o = oracle.Oracle(n, 32, 1, 0.5, 1.0, gamma=1e-6)      # threshold effectively fixed
    sel_at = None
    for t in range(6):
        o.step(g)
        if o.k_emitted:
            sel_at = t
            assert o.out_idx().tolist() == [10]
            break
    # 0.3, 0.6, 0.9 (fp32 sums) stay below 1.0; the 4th accumulation crosses it
    assert sel_at == 3
    want = np.float32(0)
    for _ in range(4):
        want = np.float32(want + np.float32(0.3))
    assert o.out_val()[0] == want
    assert o.residual()[10] == 0.0


def test_capacity_rule_truncates_in_index_order_and_keeps_the_rest():
    """This build's reading (the paper's `where` allocates freely): parity unpinned by the paper."""
    n = 1024
    rng = np.random.default_rng(5)
    g = rng.normal(0, 1, n).astype(np.float32)
    o = oracle.Oracle(n, 128, 4, 0.5, 0.1, max_selected=100)
    assert o.cap == 100
    o.step(g)
    mask = np.abs(g) >= np.float32(0.1)
    full = np.flatnonzero(mask)
    assert o.k_actual == full.size > 100 and o.k_emitted == 100
    assert np.array_equal(o.out_idx(), full[:100])
    e = o.residual()
    assert np.all(e[full[:100]] == 0) and np.array_equal(e[full[100:]], g[full[100:]])
    assert o.part_off()[-1] == 100
    assert o.part_count().sum() == full.size                # counts are untruncated
    # default capacity: max(ceil(4k), 1024) clamped to n_g
    assert oracle.Oracle(n, 128, 4, 0.5, 0.1).cap == 1024
    assert oracle.Oracle(100000, 128, 4, 0.01, 0.1).cap == 4000
    assert oracle.Oracle(100000, 128, 4, 0.001, 0.1).cap == 1024


def test_threshold_and_partial_k_feed_the_next_iteration():
    """Alg. 1 (k' sum, Estimate, partial-k carry): k' drives Estimate; this iteration's counts drive the next Allocate."""
    n, b, P = 4096, 128, 4
    rng = np.random.default_rng(11)
    # heavy head: partition 0 gets nearly all selections
    g = _rand_grad(rng, n)
    g[:512] *= 50
    o = oracle.Oracle(n, b, P, 0.02, 2e-3)
    o.step(g)
    k = 0.02 * n
    pc = o.part_count().astype(float)
    ratio = o.threshold / o.threshold_used
    exam = o.k_actual / k
    if exam > 1.1:
        assert np.isclose(ratio, 1.01, rtol=1e-6)
    assert pc[0] > pc.sum() / P and pc[1] < pc.sum() / P
    bp0 = o.blk_part(0).copy()
    o.step(_rand_grad(rng, n))
    bp1 = o.blk_part(0)
    # the overloaded partition 0 handed one block to partition 1 before selecting again
    assert bp1[0] == bp0[0] - 1
    assert bp1.sum() == bp0.sum()


def test_closed_loop_density_settles_near_target():
    """Sec. 4.4 / Sec. 5.2: the actual density is steered to the user-set density.

    Soft check on i.i.d. Laplace gradients with error feedback: after a
    warm-in (the residual has to fill up first) the selected count stays within
    a factor 1.5 of k, and the very first iteration's count is already right
    because delta_0 = s*ln(1/d) is the closed-form (1-d)-quantile of
    |Laplace(0,s)|.  The scaling has to be fine (Sec. 4.4): gamma = 0.01.
    """
    n, d, s = 200_000, 0.01, 1e-3
    w = synthetic.WORKLOADS[1].scaled(n, iters=220)
    src = synthetic.GradientSource(w, "cpu")
    o = oracle.Oracle(n, 256, 4, d, s * np.log(1 / d), gamma=0.01)
    ks = []
    for t in range(220):
        o.step(src.grad(t).numpy())
        ks.append(o.k_actual)
    k = d * n
    assert abs(ks[0] - k) < 5 * np.sqrt(k)                  # closed-form quantile
    tail = np.array(ks[100:])
    assert np.all(tail < 1.5 * k) and np.all(tail > k / 1.5)
    assert abs(tail.mean() - k) / k < 0.2


def test_hard_threshold_special_case():
    """Sec. 3: one worker and a fixed threshold is the hard-threshold sparsifier, i.e. plain
    `where(|acc| >= delta)` over the whole vector with error feedback."""
    n = 5000
    rng = np.random.default_rng(8)
    o = oracle.Oracle(n, 32, 1, 0.01, 2e-3, gamma=0.0, max_selected=n)
    e = np.zeros(n, np.float32)
    for t in range(6):
        g = _rand_grad(rng, n)
        o.step(g)
        acc = (e + g).astype(np.float32)
        sel = np.flatnonzero(np.abs(acc) >= np.float32(2e-3))
        assert np.array_equal(o.out_idx(), sel.astype(np.uint32))
        assert o.threshold == np.float32(2e-3)              # never scaled
        e = acc.copy()
        e[sel] = 0
        assert np.array_equal(o.residual(), e)


def test_stats_equations():
    """Eq. 1 (one worker), Eq. 5, Eq. 6 from their printed definitions."""
    n = 2048
    rng = np.random.default_rng(3)
    g = _rand_grad(rng, n)
    o = oracle.Oracle(n, 256, 4, 0.05, 2.5e-3)
    o.step(g)
    e = o.residual().astype(np.float64)
    assert np.isclose(o.err_norm(), np.linalg.norm(e), rtol=1e-12)
    pc = o.part_count().astype(np.float64)
    assert np.isclose(o.traffic_ratio(), 4 * pc.max() / pc.sum(), rtol=1e-15)
    assert o.traffic_ratio() >= 1.0
    assert np.isclose(o.density_error(), abs(0.05 * n - pc.sum()) / n, rtol=1e-15)


def test_rejects_bad_configurations():
    ok = dict(n_g=1024, block_size=256, n_parts=4, density=0.01, threshold0=1.0)
    oracle.Oracle(**ok)
    for bad in (dict(n_g=0), dict(block_size=0), dict(block_size=100), dict(n_parts=0),
                dict(n_parts=5), dict(density=0.0), dict(density=1.5), dict(threshold0=0.0),
                dict(threshold0=float("inf")), dict(alpha=0.5), dict(beta=1.0), dict(gamma=-0.1),
                dict(gamma=1.0), dict(min_blk=0), dict(cmp_mode=2), dict(n_g=2 ** 32)):
        with pytest.raises(ValueError):
            oracle.Oracle(**{**ok, **bad})


def _bf16_bits(x32):
    return (torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_scaled_step_rounds_product_then_sum(dtype):
    """Alg. 1 (accumulate) as printed, acc = e + eta*G: the gradient is widened exactly (checked
    against torch's bf16 and numpy's fp16 conversions), the product is rounded to fp32, then
    the sum -- numpy's separate fp32 multiply and add, never a fused multiply-add."""
    n = 3000
    rng = np.random.default_rng(40 + dtype)
    eta = np.float32(0.0371)
    o = oracle.Oracle(n, 32, 3, 0.05, 1e-4, max_selected=n)
    e = np.zeros(n, np.float32)
    for t in range(5):
        g32 = (rng.laplace(0, 1e-3, n) * 30).astype(np.float32)
        if dtype == 0:
            stored, wide = g32, g32
        elif dtype == 1:
            stored = _bf16_bits(g32)
            wide = torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).float().numpy()
        else:
            h = g32.astype(np.float16)
            h[:8] = np.array([0.0, -0.0, 6e-8, -6.1e-5, 65504.0, np.inf, -np.inf, 1e-7], np.float16)
            stored, wide = h.view(np.uint16), h.astype(np.float32)
        o.step_scaled(np.ascontiguousarray(stored), dtype, eta)
        prod = (eta * wide).astype(np.float32)
        acc = (e + prod).astype(np.float32)
        sel = np.flatnonzero(np.abs(acc) >= o.threshold_used)
        assert np.array_equal(o.out_idx(), sel.astype(np.uint32))
        assert np.array_equal(o.out_val().view(np.uint32), acc[sel].view(np.uint32))
        e = acc.copy()
        e[sel] = 0
        assert np.array_equal(o.residual().view(np.uint32), e.view(np.uint32))


def test_scaled_step_with_eta_one_equals_plain_step():
    n = 2048
    rng = np.random.default_rng(77)
    a = oracle.Oracle(n, 256, 2, 0.02, 2e-3)
    b = oracle.Oracle(n, 256, 2, 0.02, 2e-3)
    for _ in range(4):
        g = _rand_grad(rng, n)
        a.step(g)
        b.step_scaled(g, 0, 1.0)
        assert np.array_equal(a.out_idx(), b.out_idx())
        assert np.array_equal(a.residual().view(np.uint32), b.residual().view(np.uint32))
        assert a.threshold == b.threshold


def test_product_is_rounded_before_the_sum():
    """A case where fma(eta, g, e) and fl(e + fl(eta*g)) differ in the last bit."""
    eta, g, e0 = np.float32(1.4099537), np.float32(1.5942448), np.float32(-1.3154374)
    exact = float(eta) * float(g) + float(e0)                 # what a fused multiply-add rounds
    two_step = np.float32(np.float32(eta * g) + e0)
    assert np.float32(exact) != two_step
    o = oracle.Oracle(32, 32, 1, 0.5, 10.0)
    o.set_residual(np.full(32, e0, np.float32))
    o.step_scaled(np.full(32, g, np.float32), 0, eta)
    assert o.residual()[0] == two_step


def test_untruncated_counts_drive_the_threshold_and_the_next_allocate():
    """Capacity reading: what does not fit the output is still COUNTED.  Every gradient passes the
    threshold, so the four partitions hold 256 each (balanced: the next Allocate moves nothing) and
    k' = 1024 = 2k (above beta: the threshold rises); the 100 emitted pairs all lie in partition 0,
    so counts cut at the capacity would look like (100, 0, 0, 0) and a k' of 100 < k / beta."""
    n, b, P = 1024, 128, 4
    g = np.full(n, 1.0, np.float32)
    o = oracle.Oracle(n, b, P, 0.5, 0.5, gamma=0.01, beta=1.1, max_selected=100)
    o.step(g)
    assert o.k_actual == 1024 and o.k_emitted == 100
    assert o.part_count().tolist() == [256, 256, 256, 256] and o.part_off().tolist() == [0, 100, 100, 100, 100]
    assert o.threshold == np.float32(np.float32(0.5) * np.float32(1.01))      # exam = 2 > beta
    bp0 = o.blk_part(0).copy()
    o.step(np.zeros(n, np.float32))
    assert np.array_equal(o.blk_part(0), bp0) and o.blk_part(0).tolist() == [2, 2, 2, 2]


def test_fp16_nan_gradient_stays_nan_in_the_residual_and_is_never_selected():
    """Alg. 1 (accumulate) with an fp16 gradient whose bits encode a NaN (exponent all ones,
    non-zero fraction): the widened value is a NaN, so the product and the sum are NaN, Alg. 4's
    comparison is false for it, and the entry stays in the residual as a NaN on every later
    iteration.  An fp16 infinity (same exponent, zero fraction) IS selected: the two cases sit
    one fraction bit apart, so a widening that confused them fails one of the two checks."""
    n = 64
    bits = np.zeros(n, np.uint16)
    bits[3] = 0x7E00          # quiet NaN
    bits[4] = 0xFC01          # negative NaN with the lowest fraction bit only
    bits[5] = 0x7C00          # +inf
    bits[6] = 0xFC00          # -inf
    bits[7] = 0x4000          # 2.0
    assert np.isnan(bits.view(np.float16)[[3, 4]]).all() and np.isinf(bits.view(np.float16)[[5, 6]]).all()
    o = oracle.Oracle(n, 32, 2, 0.1, 1.0, max_selected=n)
    o.step_scaled(bits, 2, 1.0)
    assert o.out_idx().tolist() == [5, 6, 7]
    assert o.out_val().tolist() == [np.inf, -np.inf, 2.0]
    e = o.residual()
    assert np.isnan(e[3]) and np.isnan(e[4])
    assert np.count_nonzero(np.isnan(e)) == 2 and e[5] == 0 and e[6] == 0 and e[7] == 0
    o.step_scaled(np.zeros(n, np.uint16), 2, 1.0)           # NaN + 0 stays NaN, still not selected
    assert o.k_actual == 0 and o.k_emitted == 0
    assert np.isnan(o.residual()[[3, 4]]).all()
    assert np.isnan(o.err_norm())


def test_traffic_ratio_when_nothing_is_selected():
    """Eq. 5 is n * max_i k_i / k'; with k' = 0 it reads 0/0.  Reading taken: f(t) = 0 then (no
    traffic, nothing to balance), while Eq. 6 still gives |k - 0| / n_g."""
    n = 1024
    o = oracle.Oracle(n, 128, 4, 0.25, 10.0)
    o.step(np.full(n, 0.5, np.float32))
    assert o.k_actual == 0 and o.part_count().tolist() == [0, 0, 0, 0]
    assert o.traffic_ratio() == 0.0
    assert o.density_error() == 0.25
    assert oracle.padding_overhead(o.part_count()) == 0
    o.step(np.full(n, 20.0, np.float32))                     # everything selected, evenly: f(t) = 1
    assert o.k_actual == n and o.traffic_ratio() == 1.0
