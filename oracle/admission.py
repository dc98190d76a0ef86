"""CPU oracle of the non-blocking condition of the layer-wise fetching-inference pipeline (Appx A.3).

TEST INFRASTRUCTURE ONLY: imported by tests/ alone.  The condition is written out as the appendix states it,
one inequality per unbuffered stage k, each sum recomputed from scratch in fp64:

    for all k in {L_buf + 1, ..., L_total}:  sum_{j=1..k} T_fetch(j)  <=  sum_{j=1..k-1} T_comp(j)

(T_fetch is the appendix's per-layer decoding time: the time until the stage's KV is in the cache.)
Reading: the sums start at stage 1 as printed, also when the first L_buf stages are already buffered; a caller
whose buffered stages cost nothing more passes 0 for them.

Pins (tests marked "not gpu"): closed forms for uniform stage times, the empty constraint set (everything
buffered), monotonicity in L_buf, and a hand-evaluated four-stage example.
"""

def condition_holds(t_fetch, t_comp, n_buffered):
    """True iff every unbuffered stage's KV is ready no later than the computation of the stage before it ends."""
    n = len(t_fetch)
    assert len(t_comp) == n and n >= 1 and 0 <= n_buffered <= n
    for k in range(n_buffered + 1, n + 1):  # k is 1-based as in the appendix
        fetched = sum(float(x) for x in t_fetch[0:k])
        computed = sum(float(x) for x in t_comp[0:k - 1])
        if not fetched <= computed:
            return False
    return True


def min_buffered(t_fetch, t_comp):
    """Smallest number of buffered stages for which the condition holds (brute force over L_buf)."""
    n = len(t_fetch)
    for n_buffered in range(0, n + 1):
        if condition_holds(t_fetch, t_comp, n_buffered):
            return n_buffered
    raise AssertionError("with every stage buffered the constraint set is empty")
