"""Pins for the oracle's Alg. 2 / 3 / 5 routines: hand-evaluated fixtures and invariants.

Expectations come from tests/golden/*.json (worked by hand from the paper's
listings) or from properties the paper states (partitions never overlap and
cover the vector; cyclic ownership is a bijection), never from the oracle.
"""
import json
import os

import numpy as np
import pytest

from oracle import oracle


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


# ---------------------------------------------------------------- Alg. 2
def test_alg2_partition_hand_cases(golden_dir):
    for c in _load(golden_dir, "alg2_partition.json")["partition"]:
        bp, pos = oracle.partition(c["n_b"], c["n"])
        assert bp.tolist() == c["blk_part"], c
        assert pos.tolist() == c["blk_pos"], c


def test_alg2_quotient_remainder_of_the_five_configurations(golden_dir):
    for c in _load(golden_dir, "alg2_partition.json")["quotient_remainder"]:
        bp, pos = oracle.partition(c["n_b"], c["n"])
        assert bp[: c["r"]].tolist() == [c["q"] + 1] * c["r"]
        assert bp[c["r"]:].tolist() == [c["q"]] * (c["n"] - c["r"])
        assert int(bp.sum()) == c["n_b"]


def test_alg2_block_size_hand_cases(golden_dir):
    for c in _load(golden_dir, "alg2_partition.json")["block_size"]:
        assert oracle.block_size(c["n_g"], c["n_b"]) == c["sz_blk"], c


@pytest.mark.parametrize("seed", range(5))
def test_alg2_invariants(seed):
    rng = np.random.default_rng(seed)
    for _ in range(200):
        n = int(rng.integers(1, 70))
        n_b = int(rng.integers(n, 5000))
        bp, pos = oracle.partition(n_b, n)
        assert bp.sum() == n_b                      # every block belongs to one partition
        assert pos[0] == 0
        assert np.array_equal(pos[1:], np.cumsum(bp)[:-1])   # contiguous, non-overlapping
        assert bp.max() - bp.min() <= 1             # "equally divides"
        assert np.all(np.diff(bp) <= 0)             # the larger ones come first


# ---------------------------------------------------------------- Alg. 3
def test_alg3_sweep_hand_cases(golden_dir):
    for c in _load(golden_dir, "alg3_allocate.json")["sweep"]:
        kv, bp, pos, moves = oracle.allocate(c["k"], c["blk_part"], c["blk_pos"], c["n_g"],
                                             c["sz_blk"], c["blk_move"], c["min_blk"], c["alpha"])
        assert bp.tolist() == c["out_blk_part"], c["name"]
        assert pos.tolist() == c["out_blk_pos"], c["name"]
        assert kv.tolist() == [float(x) for x in c["out_k"]], c["name"]
        assert moves == c["moves"], c["name"]


def test_alg3_owner_hand_cases(golden_dir):
    for c in _load(golden_dir, "alg3_allocate.json")["owner"]:
        assert oracle.owner(c["t"], c["rank"], c["n"]) == c["alloc"], c


def test_alg3_owner_is_a_bijection_and_cycles():
    for n in (1, 2, 3, 8, 16, 64):
        for t in range(3 * n):
            owned = [oracle.owner(t, r, n) for r in range(n)]
            assert sorted(owned) == list(range(n))          # exclusive allocation
            for r in range(n):                              # next iteration -> next partition
                assert oracle.owner(t + 1, r, n) == (oracle.owner(t, r, n) + 1) % n


@pytest.mark.parametrize("seed", range(6))
def test_alg3_invariants_random(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(300):
        n = int(rng.integers(2, 40))
        n_b = int(rng.integers(n * 2, n * 50))
        sz = 32 * int(rng.integers(1, 64))
        n_g = n_b * sz - int(rng.integers(0, sz))
        blk_move = int(rng.integers(1, 4))
        min_blk = int(rng.integers(1, 3))
        alpha = float(rng.choice([1.0, 1.0, 1.2, 2.0]))
        bp0, pos0 = oracle.partition(n_b, n)
        # a few sweeps in a row with skewed counts
        bp, pos = bp0.copy(), pos0.copy()
        for _sweep in range(4):
            k = rng.integers(0, 1000, n).astype(np.float64) * rng.choice([1, 1, 10], n)
            kv, bp2, pos2, moves = oracle.allocate(k, bp, pos, n_g, sz, blk_move, min_blk, alpha)
            assert bp2.sum() == n_b
            assert pos2[0] == 0
            assert np.array_equal(pos2[1:], np.cumsum(bp2)[:-1])     # still a cover without overlap
            # a partition only shrinks down to min_blk, never below what it had if already below
            assert np.all(bp2 >= np.minimum(bp, min_blk))
            assert np.all(np.abs(pos2 - pos) <= blk_move)            # each boundary moves at most once
            assert np.all((pos2 - pos) % blk_move == 0)
            assert moves == int(np.count_nonzero(pos2 != pos))
            if k.sum() > 0:
                assert np.isclose(kv.sum(), k.sum(), rtol=1e-12)     # estimated counts only move around
            bp, pos = bp2, pos2


def test_alg3_moves_toward_balance():
    """Sec. 4.2: blocks go from the partition that selected more than k'/n to the one that selected less."""
    k = np.array([500.0, 20.0, 100.0, 100.0])
    bp, pos = oracle.partition(40, 4)
    _, bp2, pos2, _ = oracle.allocate(k, bp, pos, 40 * 64, 64, 1, 1, 1.0)
    assert bp2[0] == bp[0] - 1 and bp2[1] == bp[1] + 1
    k = k[::-1].copy()
    _, bp3, _, _ = oracle.allocate(k, bp, pos, 40 * 64, 64, 1, 1, 1.0)
    assert bp3[3] == bp[3] - 1 and bp3[2] == bp[2] + 1


# ---------------------------------------------------------------- Alg. 5
def test_alg5_hand_cases(golden_dir):
    for c in _load(golden_dir, "alg5_estimate.json")["cases"]:
        sf = oracle.scale_factor(c["k"], c["k_actual"], c["beta"], c["gamma"])
        assert np.float32(sf) == np.float32(float(c["sf"])), c
        for delta in (1.0, 3.0e-3, 7.25e-5):
            got = oracle.estimate(c["k"], c["k_actual"], delta, c["beta"], c["gamma"])
            want = np.float32(delta) * np.float32(float(c["sf"]))
            assert np.float32(got) == want, (c, delta)


def test_alg5_direction():
    """Sec. 4.4: more selected than required -> threshold rises; fewer -> falls."""
    k = 1000.0
    for k_act in range(0, 3000, 7):
        d1 = oracle.estimate(k, k_act, 1.0, 1.1, 0.01)
        if k_act > 1.1 * k + 1e-9:
            assert d1 > 1.0
        if k_act < k / 1.1 - 1e-9:
            assert d1 < 1.0
        assert abs(d1 - 1.0) <= 0.01 + 1e-6      # fine-grained scaling only


def test_padding_overhead_hand_cases(golden_dir):
    """Eq. 2-4 by hand (tests/golden/eq4_padding.json)."""
    for c in _load(golden_dir, "eq4_padding.json")["cases"]:
        assert max(c["k"]) == c["m_t"] and len(c["k"]) * sum(c["c"]) == c["C_t"]   # the fixture is consistent
        assert oracle.padding_overhead(c["k"]) == c["C_t"], c


def test_reindex_hand_cases(golden_dir):
    """Rank order to partition order (tests/golden/alg3_reindex.json)."""
    for c in _load(golden_dir, "alg3_reindex.json")["cases"]:
        assert oracle.reindex(c["k_rank"], c["t"]).tolist() == c["k_part"], c
