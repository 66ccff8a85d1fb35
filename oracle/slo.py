"""Oracle of the SLO-aware batching scheduler (TEST INFRASTRUCTURE ONLY).

StreamDiffusionV2, Section 4.1, "SLO-aware batching scheduler", in the paper's notation: the system processes T frames
per iteration for each of B batch slots, with inference latency L(T, B); B T must not exceed the number of frames
already collected; in the memory-bound regime
        L(T, B) ~ (A(T, B) + P_model) / (eta BW_HBM),      A(T, B) = O(B T),
and the achieved processing frequency is f = B T / L(T, B), proportional to B / (1 + B) when one slot's activation
traffic equals the parameter traffic; the scheduler settles on the batch size B* at the knee, where f stops growing.

Readings where the section is silent:
  * "satisfy the SLO" is f(B) >= f_SLO: the B T frames of an iteration are processed no slower than they arrive;
  * among the batch sizes that are allowed (B T <= frames collected) and meet the SLO, B* is the SMALLEST one whose
    frequency is within a fraction ``knee_tol`` of the best allowed frequency: past the knee a larger batch only adds
    latency.  knee_tol = 0 picks the arg-max of f (the smallest on ties);
  * if no allowed batch size meets the SLO the one with the highest frequency is returned with ``meets_slo = False``;
    if none is allowed at all (fewer than T frames collected) there is nothing to run: ``None``.
"""


def latency_model(T, B, act_bytes_per_frame, param_bytes, eta_bw):
    """L(T, B) = (A(T, B) + P_model) / (eta BW_HBM) with A(T, B) = act_bytes_per_frame * B * T; seconds."""
    return (act_bytes_per_frame * B * T + param_bytes) / eta_bw


def frequency(T, B, latency_s):
    """f = B T / L(T, B), frames per second."""
    return B * T / latency_s


def pick_batch(latency_s, T, f_slo, frames_collected, knee_tol=0.0):
    """B* from measured latencies ``latency_s`` (dict: batch size -> seconds).

    Returns None or (B*, f(B*), meets_slo)."""
    allowed = sorted(B for B in latency_s if B >= 1 and B * T <= frames_collected)
    if not allowed:
        return None
    freq = {B: frequency(T, B, latency_s[B]) for B in allowed}
    ok = [B for B in allowed if freq[B] >= f_slo]
    if not ok:
        best = max(allowed, key=lambda B: (freq[B], -B))
        return best, freq[best], False
    f_best = max(freq[B] for B in ok)
    for B in ok:                                   # ascending: the smallest one at the knee
        if freq[B] >= (1.0 - knee_tol) * f_best:
            return B, freq[B], True
    raise AssertionError("unreachable")
