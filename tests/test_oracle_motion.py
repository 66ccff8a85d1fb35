"""Pins of the motion-aware noise scheduler oracle (CPU only): the three formulas of Section 4.1 against closed forms
and explicit sums."""

import math

import numpy as np
import pytest

import oracle


def rng(seed):
    return np.random.default_rng(seed)


def test_motion_intensity_closed_forms():
    v = rng(1).normal(size=(4, 6, 5))
    assert oracle.motion_intensity(v, v) == 0.0
    assert oracle.motion_intensity(v + 0.25, v) == pytest.approx(0.25, abs=1e-15)      # constant shift c -> |c|
    assert oracle.motion_intensity(v - 3.0, v) == pytest.approx(3.0, abs=1e-14)
    w = rng(2).normal(size=(4, 6, 5))
    d = oracle.motion_intensity(v, w)
    assert oracle.motion_intensity(w, v) == pytest.approx(d, abs=1e-15)                # symmetric
    assert oracle.motion_intensity(-2.5 * v, -2.5 * w) == pytest.approx(2.5 * d, rel=1e-14)   # |a| d
    # one element differs by 1 among n: sqrt(1/n)
    z = np.zeros((2, 3, 4))
    e = z.copy()
    e[1, 2, 3] = 1.0
    assert oracle.motion_intensity(e, z) == pytest.approx(math.sqrt(1.0 / 24), abs=1e-15)
    # explicit sum
    tot = 0.0
    for a, b in zip(v.reshape(-1), w.reshape(-1)):
        tot += (float(a) - float(b)) ** 2
    assert d == pytest.approx(math.sqrt(tot / v.size), rel=1e-14)
    # mean over C H W, not a sum: doubling the frame by repetition leaves d unchanged
    assert oracle.motion_intensity(np.concatenate([v, v]), np.concatenate([w, w])) == pytest.approx(d, rel=1e-14)


def test_normalized_motion_is_window_max_over_sigma_clipped():
    assert oracle.normalized_motion([0.1, 0.4, 0.2], sigma=0.8) == pytest.approx(0.5)
    assert oracle.normalized_motion([0.1, 0.4, 0.2], sigma=0.4) == 1.0
    assert oracle.normalized_motion([0.1, 0.9], sigma=0.3) == 1.0                      # clipped above
    assert oracle.normalized_motion([0.0], sigma=2.0) == 0.0
    with pytest.raises(ValueError):
        oracle.normalized_motion([0.1], sigma=0.0)


def test_noise_rate_formula_and_limits():
    # lambda [s_max - (s_max - s_min) dhat] + (1 - lambda) s_prev
    assert oracle.noise_rate(0.5, 0.0, 0.25, 0.2, 0.9) == pytest.approx(0.25 * 0.9 + 0.75 * 0.5)
    assert oracle.noise_rate(0.5, 1.0, 0.25, 0.2, 0.9) == pytest.approx(0.25 * 0.2 + 0.75 * 0.5)
    assert oracle.noise_rate(0.5, 0.5, 0.25, 0.2, 0.9) == pytest.approx(0.25 * 0.55 + 0.75 * 0.5)
    # more motion -> lower rate (the more conservative schedule), for any previous rate
    assert oracle.noise_rate(0.7, 0.8, 0.3, 0.2, 0.9) < oracle.noise_rate(0.7, 0.1, 0.3, 0.2, 0.9)
    # the rate stays inside [s_min, s_max] when it starts there
    for dh in (0.0, 0.3, 1.0):
        assert 0.2 - 1e-15 <= oracle.noise_rate(0.2, dh, 0.4, 0.2, 0.9) <= 0.9 + 1e-15
        assert 0.2 - 1e-15 <= oracle.noise_rate(0.9, dh, 0.4, 0.2, 0.9) <= 0.9 + 1e-15


def test_static_stream_converges_geometrically_to_s_max():
    sch = oracle.MotionNoiseScheduler(k=3, sigma=1.0, lam=0.2, s_min=0.1, s_max=0.8, s_init=0.3)
    v = rng(3).normal(size=(4, 8, 8))
    for t in range(12):
        d, dh, s = sch.step(v)
        assert d == 0.0 and dh == 0.0
        assert s == pytest.approx(0.8 - (0.8 - 0.3) * (1 - 0.2) ** (t + 1), abs=1e-14)


def test_a_spike_is_held_for_k_plus_one_frames():
    k = 2
    sch = oracle.MotionNoiseScheduler(k=k, sigma=2.0, lam=0.5, s_min=0.0, s_max=1.0, s_init=1.0)
    base = np.zeros((1, 4, 4))
    frames = [base, base, base + 1.0, base + 1.0, base + 1.0, base + 1.0, base + 1.0]   # one jump at t = 2
    dhats = [sch.step(f)[1] for f in frames]
    assert dhats == [0.0, 0.0, 0.5, 0.5, 0.5, 0.0, 0.0]                                  # t = 2, 3, 4: window {t-2..t}


def test_first_frame_has_no_motion_and_the_window_is_cut_at_the_start():
    sch = oracle.MotionNoiseScheduler(k=5, sigma=1.0, lam=0.5, s_min=0.0, s_max=1.0, s_init=0.4)
    v0 = rng(4).normal(size=(2, 3, 3)) * 10
    d, dh, s = sch.step(v0)
    assert (d, dh) == (0.0, 0.0) and s == pytest.approx(0.5 * 1.0 + 0.5 * 0.4)
    v1 = v0 + 0.3
    d, dh, s1 = sch.step(v1)
    assert d == pytest.approx(0.3, abs=1e-13) and dh == pytest.approx(0.3, abs=1e-13)
    assert s1 == pytest.approx(0.5 * (1.0 - 0.3) + 0.5 * s, abs=1e-13)


def test_scheduler_against_a_brute_force_replay():
    g = rng(5)
    frames = [g.normal(size=(3, 5, 7)) * (0.2 + 0.5 * (t % 4)) for t in range(15)]
    k, sigma, lam, s_min, s_max, s0 = 3, 1.3, 0.35, 0.15, 0.85, 0.5
    sch = oracle.MotionNoiseScheduler(k, sigma, lam, s_min, s_max, s0)
    got = [sch.step(f) for f in frames]
    ds = [0.0] + [math.sqrt(sum((float(a) - float(b)) ** 2 for a, b in zip(frames[t].reshape(-1), frames[t - 1].reshape(-1)))
                            / frames[t].size) for t in range(1, 15)]
    s = s0
    for t in range(15):
        window = ds[max(0, t - k):t + 1]
        dh = min(1.0, max(0.0, max(window) / sigma))
        s = lam * (s_max - (s_max - s_min) * dh) + (1 - lam) * s
        assert got[t][0] == pytest.approx(ds[t], rel=1e-13, abs=1e-15)
        assert got[t][1] == pytest.approx(dh, rel=1e-13, abs=1e-15)
        assert got[t][2] == pytest.approx(s, rel=1e-13)
