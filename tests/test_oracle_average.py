"""Pins for oracle/average.py (paper sections 2.3, 3.2; Alg. 2; Eq. 17)."""
import os

import numpy as np
import pytest

from oracle import average

GOLD = os.path.join(os.path.dirname(__file__), "golden", "ring_rounds.txt")


def test_identical_replicas_mean_is_the_replica():
    rng = np.random.default_rng(0)
    x = rng.normal(size=37)
    for C in (1, 2):
        assert np.array_equal(average.direct_mean([x] * C), x)       # x + x and /2 are exact
    for C in (3, 4, 5, 7, 8, 16):
        # a left fold rounds from 3x on: at most C-1 roundings of 2^-53 each
        assert np.allclose(average.direct_mean([x] * C), x, rtol=C * 1.2e-16, atol=0)
    xi = np.round(x * 64.0)                                          # small integers: exact for any C
    for C in (3, 5, 8, 16):
        assert np.array_equal(average.direct_mean([xi * C] * C), xi * C)


def test_mean_is_permutation_invariant_and_matches_numpy():
    rng = np.random.default_rng(1)
    xs = [rng.normal(size=50) for _ in range(5)]
    m = average.direct_mean(xs)
    assert np.allclose(m, average.direct_mean(xs[::-1]), rtol=1e-15, atol=1e-16)
    assert np.allclose(m, np.mean(np.stack(xs), axis=0), rtol=1e-15, atol=1e-16)


@pytest.mark.parametrize("C", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("R", [1, 2, 3, 4])
def test_ring_equals_direct_mean_brute_force(C, R):
    rng = np.random.default_rng(100 * C + R)
    for n in list(range(1, 41, 3)) + [R * C - 1 if R * C > 1 else 1, 64]:
        # small integers scaled by C: every partial sum and the division are exact in fp64
        xs = [rng.integers(-50, 50, size=n).astype(np.float64) * C for _ in range(C)]
        bufs, rounds, sent = average.multi_ring_allreduce(xs, R)
        ref = average.direct_mean(xs)
        assert rounds == 2 * (C - 1)
        for b in bufs:                                   # every cluster ends with the mean
            assert np.array_equal(b, ref)
        xr = [rng.normal(size=n) for _ in range(C)]
        bufs, _, _ = average.multi_ring_allreduce(xr, R)
        assert np.allclose(bufs[0], average.direct_mean(xr), rtol=0, atol=1e-15)


def test_round_count_printed_in_paper():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        devices, rounds = map(int, line.split())
        _, r, _ = average.multi_ring_allreduce([np.zeros(12)] * devices, 1)
        assert r == rounds


def test_sent_elements_closed_form():
    # per ring and per replica 2(C-1) * S_r / C elements when C divides S_r
    C, R, n = 4, 3, 3 * 4 * 5
    xs = [np.arange(n, dtype=np.float64) + c for c in range(C)]
    _, _, sent = average.multi_ring_allreduce(xs, R)
    for r in range(R):
        assert sent[r] == [2 * (C - 1) * (n // R) // C] * C


def test_partition_covers_vector_once():
    for n, R, C in [(10, 3, 4), (5, 4, 3), (64, 2, 16), (1, 1, 1), (7, 8, 2)]:
        b = average.ring_partition(n, R, C)
        flat = [(b[r][j], b[r][j + 1]) for r in range(R) for j in range(C)]
        assert flat[0][0] == 0 and flat[-1][1] == n
        assert all(flat[i][1] == flat[i + 1][0] for i in range(len(flat) - 1))
        assert all(lo <= hi for lo, hi in flat)


def test_fused_update_moves_mean_by_eta_g_over_C():
    rng = np.random.default_rng(2)
    C, n, eta = 4, 33, 0.25
    xs = [rng.integers(-8, 8, size=n).astype(np.float64) for _ in range(C)]
    g = rng.integers(-8, 8, size=n).astype(np.float64)
    for cstar in range(C):
        m = average.direct_mean(xs, g, cstar, eta)
        assert np.array_equal(m - average.direct_mean(xs), -(eta / C) * g)     # Eq. 17
        bufs, _, _ = average.multi_ring_allreduce(xs, 2, g, cstar, eta)
        assert np.array_equal(bufs[cstar], m)


@pytest.mark.parametrize("C,R,n", [(2, 2, 101), (3, 2, 64), (4, 4, 257), (16, 8, 1000), (5, 3, 7)])
def test_fp32_ring_order_twin_matches_fp32_simulation_bitwise(C, R, n):
    rng = np.random.default_rng(3)
    xs = [rng.normal(size=n).astype(np.float32) for _ in range(C)]
    g = rng.normal(size=n).astype(np.float32)
    bufs, _, _ = average.multi_ring_allreduce(xs, R, g, 1 % C, 1e-2, dtype=np.float32)
    twin = average.ring_order_mean_f32(xs, R, g, 1 % C, 1e-2)
    assert twin.dtype == np.float32
    assert np.array_equal(bufs[0], twin) and np.array_equal(bufs[C - 1], twin)
    ref = average.direct_mean(xs, g, 1 % C, 1e-2)
    bound = 1e-6 * (np.mean(np.abs(np.stack(xs)), axis=0) + 1e-2 * np.abs(g) / C)
    assert np.all(np.abs(twin.astype(np.float64) - ref) <= bound)


@pytest.mark.parametrize("C", [2, 3, 4])
def test_unequal_rings_equal_direct_mean(C):
    """Rings of unequal size (explicit boundaries): still the plain mean, 2(C-1) rounds, and
    the equal-split table reproduces the default partition."""
    rng = np.random.default_rng(7 + C)
    n = 61
    for offs in ([0, 5, 5, 40, 61], [0, 1, 61], [0, 61], [0, 0, 30, 61], [0, 20, 41, 60, 61]):
        R = len(offs) - 1
        xs = [rng.integers(-50, 50, size=n).astype(np.float64) * C for _ in range(C)]
        bufs, rounds, sent = average.multi_ring_allreduce(xs, R, ring_offsets=offs)
        assert rounds == 2 * (C - 1)
        ref = average.direct_mean(xs)
        for b in bufs:
            assert np.array_equal(b, ref)
        flat = [x for rb in average.ring_partition(n, R, C, offs) for x in zip(rb[:-1], rb[1:])]
        assert flat[0][0] == 0 and flat[-1][1] == n and all(a[1] == b[0] for a, b in zip(flat, flat[1:]))
        x32 = [x.astype(np.float32) for x in xs]
        b32, _, _ = average.multi_ring_allreduce(x32, R, dtype=np.float32, ring_offsets=offs)
        assert np.array_equal(b32[0], average.ring_order_mean_f32(x32, R, ring_offsets=offs))
    eq = [(r * n) // 4 for r in range(5)]
    assert average.ring_partition(n, 4, C, eq) == average.ring_partition(n, 4, C)
