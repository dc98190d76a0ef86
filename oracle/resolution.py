"""CPU oracle of the adaptive-resolution selector (Alg. 1, Appx A.2; Sec. 3.3.1 bandwidth-aware adaptation).

TEST INFRASTRUCTURE ONLY: imported by tests/ alone.  The steps are taken in the algorithm's order and notation:
predict the bandwidth, then for every supported resolution r compute the transmission latency S_r / B, look up the
decoding latency for the present pool load and the switching penalty, form the bubble |tau_trans - tau_dec -
tau_penalty| and keep the resolution with the smallest bubble (a later resolution replaces the kept one only if its
bubble is strictly smaller).

Readings: the penalty is charged only when r differs from the resolution the decode pool is working on (text below
the algorithm); an idle pool (active = -1) has nothing to switch from; the bandwidth predictor is the simple one the
paper names: size of the last chunk over its transmission delay.

Pins (tests marked "not gpu"): the three lookup tables the paper prints with hand-evaluated selections
(tests/golden/alg1_*.txt), the zero-bubble case, the tie rule, invariance under a common scaling of all times.
"""


def est_bandwidth(last_chunk_size, last_transmission_delay):
    """Bandwidth predicted from the last chunk alone."""
    return float(last_chunk_size) / float(last_transmission_delay)


def select_resolution(sizes, latency, penalty, pool_load, active, bandwidth):
    """sizes[r], penalty[r]; latency[load - 1][r] as the paper's tables are printed (one row per concurrency).
    Returns (r_opt, bubble)."""
    n = len(sizes)
    assert len(penalty) == n and 1 <= pool_load <= len(latency) and -1 <= active < n and bandwidth > 0
    delta_min = float("inf")
    r_opt = None
    for r in range(n):
        tau_trans = float(sizes[r]) / float(bandwidth)
        tau_dec = float(latency[pool_load - 1][r])
        tau_penalty = float(penalty[r]) if (active != -1 and r != active) else 0.0
        delta_bubble = abs(tau_trans - tau_dec - tau_penalty)
        if delta_bubble < delta_min:
            delta_min = delta_bubble
            r_opt = r
    return r_opt, delta_min
