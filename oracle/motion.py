"""Oracle of the motion-aware noise scheduler (TEST INFRASTRUCTURE ONLY).

StreamDiffusionV2, Section 4.1, "Motion-aware noise scheduler", in the paper's notation:
  * motion intensity between consecutive latent frames v_t, v_{t-1} in R^{C x H x W}:
        d_t = sqrt( ||v_t - v_{t-1}||_2^2 / (C H W) );
  * normalised over a short window of k frames by a scale sigma and clipped:
        dhat_t = clip( max_{i in {t-k, ..., t}} d_i / sigma, 0, 1 );
  * noise rate smoothed by an exponential moving average:
        s_t = lambda [ s_max - (s_max - s_min) dhat_t ] + (1 - lambda) s_{t-1},   0 < lambda < 1.

Readings where the section is silent:
  * the first frame of a stream has no predecessor: d_0 = 0;
  * the window {t-k, ..., t} holds k + 1 values and is cut at the start of the stream (frames before 0 do not exist);
  * s_{-1}, the rate before the first frame, is a parameter (``s_init``).

Plain float64, one frame at a time; nothing here is shared with the HIP library.
"""

import math

import numpy as np


def motion_intensity(v_t, v_prev):
    """d_t: root mean square of the element-wise difference of two latent frames of equal shape."""
    a = np.asarray(v_t, dtype=np.float64).reshape(-1)
    b = np.asarray(v_prev, dtype=np.float64).reshape(-1)
    if a.shape != b.shape or a.size == 0:
        raise ValueError("frames must have the same, non-zero size")
    diff = a - b
    return math.sqrt(float(np.dot(diff, diff)) / a.size)


def normalized_motion(d_window, sigma):
    """dhat_t from the d values of frames t-k .. t (however many exist) and the scale sigma."""
    if sigma <= 0:
        raise ValueError("sigma must be positive")
    m = max(d_window) / sigma
    return min(max(m, 0.0), 1.0)


def noise_rate(s_prev, d_hat, lam, s_min, s_max):
    """s_t = lambda [s_max - (s_max - s_min) dhat_t] + (1 - lambda) s_{t-1}."""
    return lam * (s_max - (s_max - s_min) * d_hat) + (1.0 - lam) * s_prev


class MotionNoiseScheduler:
    """The recurrence over a stream of latent frames."""

    def __init__(self, k, sigma, lam, s_min, s_max, s_init):
        if k < 0 or not 0.0 < lam < 1.0 or s_min > s_max:
            raise ValueError("bad parameters")
        self.k, self.sigma, self.lam = int(k), float(sigma), float(lam)
        self.s_min, self.s_max = float(s_min), float(s_max)
        self.s = float(s_init)
        self.d_hist = []            # every d_t so far (the window is its last k + 1 entries)
        self.prev = None

    def step(self, v_t):
        """Feed frame v_t; returns (d_t, dhat_t, s_t)."""
        v = np.asarray(v_t, dtype=np.float64)
        d = 0.0 if self.prev is None else motion_intensity(v, self.prev)
        self.prev = v.copy()
        self.d_hist.append(d)
        d_hat = normalized_motion(self.d_hist[-(self.k + 1):], self.sigma)
        self.s = noise_rate(self.s, d_hat, self.lam, self.s_min, self.s_max)
        return d, d_hat, self.s
