"""Pins of the SLO-aware batching scheduler oracle (CPU only)."""

import itertools

import numpy as np
import pytest

import oracle


def test_latency_model_and_the_b_over_one_plus_b_law():
    # when one slot's activation traffic equals the parameter traffic, f is proportional to B / (1 + B)
    T, a, eta_bw = 4, 2.5e8, 3.0e12
    P = a * T
    f = [oracle.frequency(T, B, oracle.latency_model(T, B, a, P, eta_bw)) for B in range(1, 9)]
    ratios = [f[B - 1] / (B / (1.0 + B)) for B in range(1, 9)]
    assert max(ratios) - min(ratios) <= 1e-9 * ratios[0]
    assert ratios[0] == pytest.approx(eta_bw / a, rel=1e-12)                   # the constant: eta BW / bytes per frame
    assert all(f[i] < f[i + 1] for i in range(7)) and f[7] < eta_bw / a        # rising, bounded by the compute-free limit
    # latency is affine in B with the parameter term as the intercept
    L = [oracle.latency_model(T, B, a, P, eta_bw) for B in (0, 1, 2)]
    assert L[0] == pytest.approx(P / eta_bw) and L[2] - L[1] == pytest.approx(L[1] - L[0])


def test_pick_batch_constraints_and_knee():
    T = 2
    lat = {1: 0.010, 2: 0.012, 4: 0.016, 8: 0.030, 16: 0.060}                 # f = 200, 333, 500, 533, 533
    # everything allowed, SLO low: arg-max of f, the smaller batch on the tie
    assert oracle.pick_batch(lat, T, 100.0, 1000) == (8, pytest.approx(533.333333), True)
    # a knee tolerance of 10 %: B = 4 is within 10 % of the best and comes first
    assert oracle.pick_batch(lat, T, 100.0, 1000, knee_tol=0.10)[0] == 4
    # frames collected bound B T
    assert oracle.pick_batch(lat, T, 100.0, 9)[0] == 4
    assert oracle.pick_batch(lat, T, 100.0, 3)[0] == 1
    assert oracle.pick_batch(lat, T, 100.0, 1) is None
    # an SLO that only the large batches meet
    assert oracle.pick_batch(lat, T, 510.0, 1000, knee_tol=0.5)[0] == 8
    # an SLO nobody meets: best effort, flagged
    B, f, ok = oracle.pick_batch(lat, T, 1000.0, 9)
    assert (B, ok) == (4, False) and f == pytest.approx(500.0)


def test_pick_batch_against_brute_force():
    g = np.random.default_rng(0)
    for trial in range(300):
        sizes = sorted(g.choice(np.arange(1, 20), size=int(g.integers(1, 7)), replace=False).tolist())
        lat = {B: float(g.uniform(0.5, 3.0)) * (0.3 + B) * 1e-3 for B in sizes}
        T = int(g.integers(1, 5))
        f_slo = float(g.uniform(100, 3000))
        frames = int(g.integers(0, 60))
        tol = float(g.choice([0.0, 0.05, 0.2]))
        got = oracle.pick_batch(lat, T, f_slo, frames, tol)
        allowed = [B for B in sizes if B * T <= frames]
        if not allowed:
            assert got is None
            continue
        f = {B: B * T / lat[B] for B in allowed}
        ok = [B for B in allowed if f[B] >= f_slo]
        if not ok:
            top = max(f.values())
            assert got[2] is False and f[got[0]] == top and got[0] == min(B for B in allowed if f[B] == top)
            continue
        top = max(f[B] for B in ok)
        want = min(B for B in ok if f[B] >= (1 - tol) * top)
        assert got == (want, pytest.approx(f[want]), True)
